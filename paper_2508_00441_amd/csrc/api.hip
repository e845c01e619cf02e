// C ABI of libozaki: contexts, argument checks, the planner (Eq. 1-3), workspace carve-up and the kernel sequence.
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "../../include/ozaki_dgemm.h"
#include "layout.hpp"

using namespace ozaki;

static_assert(OZAKI_MAX_SLICES == MAX_SLICES, "header and implementation disagree");
static_assert(OZAKI_SLICE_INT8 == FMT_INT8 && OZAKI_ACCUM_EXACT_FIXED == ACC_EXACT && OZAKI_SUM_PLAIN == SUM_PLAIN,
              "header and implementation disagree");

// A context: everything a call needs beyond its arguments.
struct ozaki_context_s {
    hipStream_t stream = nullptr;
    uint8_t* ws = nullptr;
    size_t ws_bytes = 0;
    int last_hip_error = 0;
    bool profiling = false;
    struct Span { hipEvent_t e0, e1; int phase; };
    std::vector<Span> spans;       // recorded since the last ozaki_profile_read
    std::vector<hipEvent_t> pool;  // idle events
};

namespace {

typedef ozaki_context_s Context;

Context default_context;
thread_local Context* current_context = nullptr;
Context& ctx() { return current_context ? *current_context : default_context; }

constexpr size_t MAX_SPANS = 4096;

// Work memory of ozaki_dgemm_static: one array per GPU the library runs on, part of the loaded code object (zero when
// the object is loaded), so that the entry point never allocates.  Host code must not use the array's name as an
// address: the per-device address comes from hipGetSymbolAddress, once per device, and is kept in static_scratch_ptr.
static __device__ __align__(256) unsigned char static_scratch[OZAKI_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
uint8_t* static_scratch_ptr[MAX_DEVICES] = {};

constexpr size_t ALIGN = 256;
constexpr size_t FLAG_BYTES = 256;
constexpr size_t P_BUDGET = (size_t)160 << 30;        // resident pair products: well inside the 288 GB of one GPU
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

int fail_hip(hipError_t e) {
    ctx().last_hip_error = (int)e;
    return OZAKI_STATUS_HIP_ERROR;
}
#define HIP_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return fail_hip(e_); } while (0)

// Exact window of the matrix unit's accumulator, in units of the product of two slice units: |sum| <= window is exact.
int64_t exact_window(int fmt) { return fmt == OZAKI_SLICE_INT8 ? ((int64_t)1 << 31) - 1 : (int64_t)1 << 24; }

// Largest b <= m2 with kb * 4^b <= window (Eq. 1-3 with Type1 = FP64, Type3 = FP32 / INT32); -1 if none.
int slice_bits(int64_t kb, int fmt) {
    // significand bits with the hidden one: E4M3 and E2M3 have three fraction bits, E3M2 two; an INT8 byte holds |q| <= 2^6
    const int m2 = fmt == OZAKI_SLICE_FP16 ? 11 : fmt == OZAKI_SLICE_FP6_E3M2 ? 3 : fmt == OZAKI_SLICE_INT8 ? 6 : 4;
    const int64_t window = exact_window(fmt);
    for (int b = m2; b >= 0; --b)
        if (kb <= (window >> (2 * b))) return b;
    return -1;
}

bool format_ok(int fmt) { return fmt >= OZAKI_SLICE_FP8_E4M3 && fmt <= OZAKI_SLICE_INT8; }

// Builds the plan; returns 0 or a status / negative argument index in the numbering of ozaki_dgemm.
int make_plan(int64_t m, int64_t n, int64_t k, int fmt, int s, int64_t k_block, bool full, Plan& pl) {
    if (m < 0) return -1;
    if (n < 0) return -2;
    if (k < 0) return -3;
    if (!format_ok(fmt)) return -10;
    if (s < 0) return -11;
    if (k_block < 0) return -12;
    memset(&pl, 0, sizeof(pl));
    pl.m = m; pl.n = n; pl.k = k; pl.fmt = fmt;
    pl.epc = fmt == OZAKI_SLICE_FP16 ? CHUNK_BYTES / 2 : CHUNK_BYTES;
    pl.row_bytes = fmt_is_fp6(fmt) ? CHUNK_BYTES_FP6 : CHUNK_BYTES;
    pl.kb = (k_block == 0 || k_block > k) ? k : k_block;
    if (pl.kb < 1) pl.kb = 1;
    pl.b = slice_bits(pl.kb, fmt);
    if (pl.b < 0) return OZAKI_STATUS_INFEASIBLE;
    pl.rho = 53 - pl.b;
    pl.s = s == 0 ? (61 + pl.b) / (pl.b + 1) : s;
    if (pl.s > MAX_SLICES) return OZAKI_STATUS_SLICE_COUNT;
    pl.T = k == 0 ? 0 : (k + pl.kb - 1) / pl.kb;
    pl.p_frac = 2 * pl.b - (fmt == OZAKI_SLICE_FP6_E2M3 ? 2 : 0);
    pl.p_is_int = fmt == OZAKI_SLICE_INT8 ? 1 : 0;
    if (pl.p_is_int) pl.p_frac = 0;               // the stored words are the integers themselves
    pl.chunks = (pl.kb + pl.epc - 1) / pl.epc;
    pl.full = full ? 1 : 0;
    pl.npairs = full ? pl.s * pl.s : pl.s * (pl.s + 1) / 2;
    const int64_t rl = exact_window(fmt) / (pl.kb << (2 * pl.b));
    pl.run_limit = rl < 1 ? 1 : rl > MAX_SLICES ? MAX_SLICES : (int)rl;
    pl.tiles_m = (m + TILE - 1) / TILE;
    pl.tiles_n = (n + TILE - 1) / TILE;
    pl.m_pad = pl.tiles_m * TILE;
    pl.n_pad = pl.tiles_n * TILE;
    // Length of the GEMM kernel's groups.  Any length up to run_limit gives the same bits (the accumulation kernel
    // merges equal-scale products of an anti-diagonal element by element whatever the grouping).  Long groups store
    // fewer products; shorter ones give a problem of few tiles enough workgroups to keep 256 compute units evenly
    // busy, which pays once a pair streams at least 64 stages, so that one more product store per group is small
    // against it (measured at 16 tiles, 128 stages: 17 ... 28 % less GEMM time at 560 instead of 288 workgroups).
    pl.group_len = pl.run_limit;
    if (pl.chunks >= 64)
        while (pl.group_len > 2 && pl.tiles_m * pl.tiles_n * order_num_groups(PairOrder{pl.s, pl.full, pl.group_len}) < 512) --pl.group_len;
    return 0;
}

struct WorkMem {
    uint8_t* ptr;
    size_t bytes;
};

struct Carve {
    int* flags;
    double* At;
    void* split_state;    // per-element state of the streaming slicing kernel (long blocks only)
    Operand A, B;
    double* W;            // m x n product buffer of the scaled call (null otherwise)
    uint64_t* S;
    float* P;
    int chunk_pairs;
};

size_t slices_bytes(const Plan& pl, int64_t rows_pad) { return align_up((size_t)pl.T * pl.s * pl.chunks * rows_pad * pl.row_bytes); }
size_t exps_bytes(const Plan& pl, int64_t rows_pad) { return align_up((size_t)pl.T * pl.s * rows_pad * sizeof(int32_t)); }
size_t deltas_bytes(const Plan& pl, int64_t rows_pad) { return align_up((size_t)pl.T * (rows_pad / LINK_ROWS) * pl.s * sizeof(int32_t)); }
size_t state_bytes(const Plan& pl) { return align_up(split_state_bytes(pl, pl.m, pl.n)); }
size_t fixed_bytes(const Plan& pl) {
    return FLAG_BYTES + align_up((size_t)pl.m * pl.k * sizeof(double)) + state_bytes(pl) + slices_bytes(pl, pl.m_pad) +
           slices_bytes(pl, pl.n_pad) + exps_bytes(pl, pl.m_pad) + exps_bytes(pl, pl.n_pad) + deltas_bytes(pl, pl.m_pad) +
           deltas_bytes(pl, pl.n_pad);
}
size_t pair_bytes(const Plan& pl) { return (size_t)pl.m_pad * pl.n_pad * sizeof(float); }
// running block sum between passes: room for the three words of the exact mode whatever the mode
size_t sum_bytes(const Plan& pl) { return (size_t)pl.m_pad * pl.n_pad * sizeof(uint64_t) * SUM_WORDS_MAX; }

size_t recommended_bytes(const Plan& pl) {
    const size_t all = (size_t)pl.npairs * pair_bytes(pl);
    if (all <= P_BUDGET) return fixed_bytes(pl) + all;
    size_t fit = P_BUDGET / pair_bytes(pl);
    if (fit < (size_t)pl.s) fit = pl.s;
    return fixed_bytes(pl) + sum_bytes(pl) + fit * pair_bytes(pl);
}
// The pair list is processed in passes that end at anti-diagonal boundaries (a run of equal-scale products
// never spans two passes), so the smallest workspace holds the longest anti-diagonal: s products.
size_t minimum_bytes(const Plan& pl) {
    if (pl.npairs == 1) return fixed_bytes(pl) + pair_bytes(pl);
    return fixed_bytes(pl) + sum_bytes(pl) + (size_t)pl.s * pair_bytes(pl);
}

size_t product_bytes(const Plan& pl) { return align_up((size_t)pl.m * pl.n * sizeof(double)); }

// Places every buffer in the work memory; returns false if it does not fit.
bool carve(const Plan& pl, Carve& c, bool want_product, WorkMem wm) {
    uint8_t* const ws = wm.ptr;
    const size_t ws_bytes = wm.bytes;
    if (!ws) return false;
    size_t off = 0;
    c.flags = reinterpret_cast<int*>(ws);
    off += FLAG_BYTES;
    c.At = reinterpret_cast<double*>(ws + off);
    off += align_up((size_t)pl.m * pl.k * sizeof(double));
    c.split_state = state_bytes(pl) ? ws + off : nullptr;
    off += state_bytes(pl);
    c.A.rows = pl.m; c.A.rows_pad = pl.m_pad;
    c.B.rows = pl.n; c.B.rows_pad = pl.n_pad;
    c.A.slices = ws + off; off += slices_bytes(pl, pl.m_pad);
    c.B.slices = ws + off; off += slices_bytes(pl, pl.n_pad);
    c.A.exps = reinterpret_cast<int32_t*>(ws + off); off += exps_bytes(pl, pl.m_pad);
    c.B.exps = reinterpret_cast<int32_t*>(ws + off); off += exps_bytes(pl, pl.n_pad);
    c.A.deltas = reinterpret_cast<int32_t*>(ws + off); off += deltas_bytes(pl, pl.m_pad);
    c.B.deltas = reinterpret_cast<int32_t*>(ws + off); off += deltas_bytes(pl, pl.n_pad);
    c.W = nullptr;
    if (want_product) { c.W = reinterpret_cast<double*>(ws + off); off += product_bytes(pl); }
    if (off > ws_bytes) return false;
    const size_t rest = ws_bytes - off, pb = pair_bytes(pl);
    if (pb == 0) { c.S = nullptr; c.P = nullptr; c.chunk_pairs = pl.npairs; return true; }
    if (rest >= (size_t)pl.npairs * pb) {
        c.S = nullptr;
        c.P = reinterpret_cast<float*>(ws + off);
        c.chunk_pairs = pl.npairs;
        return true;
    }
    if (rest < sum_bytes(pl) + (size_t)pl.s * pb) return false;
    c.S = reinterpret_cast<uint64_t*>(ws + off);
    off += sum_bytes(pl);
    c.P = reinterpret_cast<float*>(ws + off);
    size_t fit = (ws_bytes - off) / pb;
    c.chunk_pairs = fit > (size_t)pl.npairs ? pl.npairs : (int)fit;
    return c.chunk_pairs >= pl.s;
}

PairOrder order_of(const Plan& pl) { return PairOrder{pl.s, pl.full, pl.group_len}; }

// The pass that starts at anti-diagonal g_hi: as many whole anti-diagonals as fit into `capacity` products (at
// least one: the carve-up guarantees room for the longest anti-diagonal).
Pass next_pass(const PairOrder& o, int g_hi, int capacity) {
    Pass ps{g_hi, g_hi, 0, 0};
    for (int g = g_hi; g >= 2; --g) {
        const int len = diag_len(o, g);
        if (ps.npairs > 0 && ps.npairs + len > capacity) break;
        ps.g_lo = g;
        ps.npairs += len;
        ps.ngroups += diag_groups(o, g);
    }
    return ps;
}

// ---- profiling spans -------------------------------------------------------------------------------------------
hipEvent_t take_event(Context& c) {
    hipEvent_t e = nullptr;
    if (!c.pool.empty()) { e = c.pool.back(); c.pool.pop_back(); return e; }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
// Brackets a phase with two events when profiling is on, the span list has room and the stream is not being
// captured into a graph (events recorded under capture cannot be timed).
struct Phase {
    Context& c;
    int phase; hipEvent_t e0 = nullptr, e1 = nullptr;
    explicit Phase(int ph) : c(ctx()), phase(ph) {
        if (!c.profiling || c.spans.size() >= MAX_SPANS) return;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(c.stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return;
        e0 = take_event(c);
        e1 = e0 ? take_event(c) : nullptr;
        if (!e1) {                                       // no second event: give the first one back
            if (e0) c.pool.push_back(e0);
            e0 = nullptr;
            return;
        }
        (void)hipEventRecord(e0, c.stream);
    }
    ~Phase() {
        if (!e0 || !e1) return;
        (void)hipEventRecord(e1, c.stream);
        c.spans.push_back({e0, e1, phase});
    }
};

// split both operands of the plan into the carved buffers
int run_split(const Plan& pl, const Carve& c, const double* A, int64_t lda, const double* B, int64_t ldb, bool do_a, bool do_b) {
    Phase ph(0);
    hipStream_t st = ctx().stream;
    const bool a_on = do_a && pl.m > 0, b_on = do_b && pl.n > 0;
    if (a_on) HIP_TRY(launch_transpose(A, lda, pl.m, pl.k, c.At, st));
    // both operands in one launch each: on a small problem neither fills the chip alone
    HIP_TRY(launch_split(c.At, pl.k, a_on ? &c.A : nullptr, B, ldb, b_on ? &c.B : nullptr, pl, c.flags, c.split_state, st));
    HIP_TRY(launch_deltas(pl, a_on ? &c.A : nullptr, b_on ? &c.B : nullptr, st));
    return 0;
}

// zeros and normal numbers only: what the emulated multiplication covers (Section 4.2)
bool scalar_ok(double v) {
    uint64_t b;
    memcpy(&b, &v, 8);
    const int e = (int)((b >> 52) & 0x7FF);
    return (e != 0 && e != 0x7FF) || (b << 1) == 0;
}

struct Options {
    int slice_format, num_slices;
    int64_t k_block;
    int accum_mode, pair_set, sum_rule;
};

// Argument checks shared by the DGEMM entry points (positions of ozaki_dgemm / ozaki_dgemm_ex).
int check_dgemm_args(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                     const double* C, int64_t ldc, const Options& o, Plan& pl) {
    if (o.pair_set != OZAKI_PAIRS_TRIANGLE && o.pair_set != OZAKI_PAIRS_ALL) return -14;
    const int st = make_plan(m, n, k, o.slice_format, o.num_slices, o.k_block, o.pair_set == OZAKI_PAIRS_ALL, pl);
    if (st != 0) return st;
    if (o.accum_mode < OZAKI_ACCUM_FP64_HW || o.accum_mode > OZAKI_ACCUM_EXACT_FIXED) return -13;
    if (o.sum_rule != OZAKI_SUM_RUNS && o.sum_rule != OZAKI_SUM_PLAIN) return -15;
    if (m == 0 || n == 0) return 0;
    if (!C) return -8;
    if (ldc < (m > 1 ? m : 1)) return -9;
    if (k > 0) {
        if (!A) return -4;
        if (lda < (m > 1 ? m : 1)) return -5;
        if (!B) return -6;
        if (ldb < (k > 1 ? k : 1)) return -7;
    }
    return 0;
}

// One Ozaki product on (a panel of) the operands: C = alpha * (A B) + beta * C.  (alpha, beta) = (1, 0): the product
// goes straight to C.  Otherwise it goes to the work memory's product buffer and one more kernel combines it with C.
// The arguments have been checked and the plan made (check_dgemm_args).
int dgemm_core(const Plan& pl, double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C,
               int64_t ldc, const Options& o, WorkMem wm) {
    const int64_t m = pl.m, n = pl.n, k = pl.k;
    if (m == 0 || n == 0) return 0;
    hipStream_t st = ctx().stream;
    const bool scaled = !(alpha == 1.0 && beta == 0.0);
    Carve c;
    c.W = nullptr;
    if ((k > 0 || scaled) && !carve(pl, c, scaled, wm)) return OZAKI_STATUS_WORKSPACE;
    double* const out = scaled ? c.W : C;
    const int64_t ldo = scaled ? (m > 1 ? m : 1) : ldc;
    if (k == 0) {
        HIP_TRY(launch_fill_zero_f64(out, ldo, m, n, st));
    } else {
        const PairOrder order = order_of(pl);
        // the plain rule adds every product on its own, so the matrix unit must not sum across pairs
        const bool chained = o.sum_rule == OZAKI_SUM_RUNS || o.accum_mode == OZAKI_ACCUM_EXACT_FIXED;
        int rc = run_split(pl, c, A, lda, B, ldb, true, true);
        if (rc) return rc;
        for (int64_t t = 0; t < pl.T; ++t) {
            for (int g_hi = order_top_diag(order); g_hi >= 2;) {
                const Pass ps = next_pass(order, g_hi, c.chunk_pairs);
                {
                    Phase ph(1);
                    HIP_TRY(launch_pair_gemm(pl, c.A, c.B, order, ps, chained, t, c.P, st));
                }
                {
                    Phase ph(2);
                    HIP_TRY(launch_accumulate(pl, c.A, c.B, order, ps, g_hi == order_top_diag(order), ps.g_lo == 2, t, c.P, c.S, out,
                                              ldo, o.accum_mode, o.sum_rule, chained, st));
                }
                g_hi = ps.g_lo - 1;
            }
        }
    }
    if (scaled) {
        Phase ph(2);
        HIP_TRY(launch_axpby(alpha, beta, c.W, ldo, C, ldc, m, n, o.accum_mode != OZAKI_ACCUM_FP64_HW, st));
    }
    return 0;
}

// Outer-product-wise blocking (Section 4.3): panels of rows of A times panels of columns of B, each an Ozaki product
// of its own inside the capped work memory.  Rows of A and columns of B are sliced independently of the rest
// of their matrices, so every panel product carries the bits of the unblocked call.
int dgemm_panels(const Plan& whole, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                 const Options& o, WorkMem wm) {
    int64_t mb = whole.m_pad, nb = whole.n_pad;
    Plan pl;
    for (;;) {
        const int st = make_plan(mb < whole.m ? mb : whole.m, nb < whole.n ? nb : whole.n, whole.k, o.slice_format, whole.s, o.k_block,
                                 whole.full != 0, pl);
        if (st != 0) return st;
        if (minimum_bytes(pl) <= wm.bytes) break;
        if (mb <= TILE && nb <= TILE) return OZAKI_STATUS_WORKSPACE;
        int64_t& big = mb >= nb ? mb : nb;                 // halve the longer side, in whole tiles
        big = ((big / TILE + 1) / 2) * TILE;
    }
    for (int64_t i0 = 0; i0 < whole.m; i0 += mb)
        for (int64_t j0 = 0; j0 < whole.n; j0 += nb) {
            const int64_t mi = whole.m - i0 < mb ? whole.m - i0 : mb, nj = whole.n - j0 < nb ? whole.n - j0 : nb;
            const int st = make_plan(mi, nj, whole.k, o.slice_format, whole.s, o.k_block, whole.full != 0, pl);
            if (st != 0) return st;
            const int rc = dgemm_core(pl, 1.0, A + i0, lda, B + j0 * ldb, ldb, 0.0, C + i0 + j0 * ldc, ldc, o, wm);
            if (rc != 0) return rc;
        }
    return 0;
}

WorkMem context_workspace() { return WorkMem{ctx().ws, ctx().ws_bytes}; }

int plan_for_query(int64_t m, int64_t n, int64_t k, int fmt, int s, int64_t k_block, int pair_set, Plan& pl) {
    if (pair_set != OZAKI_PAIRS_TRIANGLE && pair_set != OZAKI_PAIRS_ALL) return -14;
    return make_plan(m, n, k, fmt, s, k_block, pair_set == OZAKI_PAIRS_ALL, pl);
}

}  // namespace

extern "C" {

int ozaki_context_create(ozaki_context_t* ctx_out) {
    if (!ctx_out) return -1;
    *ctx_out = new (std::nothrow) ozaki_context_s();
    return *ctx_out ? 0 : OZAKI_STATUS_HIP_ERROR;
}

int ozaki_context_destroy(ozaki_context_t c) {
    if (!c || c == &default_context) return -1;
    if (current_context == c) current_context = nullptr;
    for (auto& sp : c->spans) { (void)hipEventDestroy(sp.e0); (void)hipEventDestroy(sp.e1); }
    for (auto e : c->pool) (void)hipEventDestroy(e);
    delete c;
    return 0;
}

int ozaki_context_use(ozaki_context_t c) {
    current_context = (c == &default_context) ? nullptr : c;
    return 0;
}

int ozaki_plan(int64_t k_block, int slice_format, int* rho_out, int* bits_out) {
    if (k_block < 1) return -1;
    if (!format_ok(slice_format)) return -2;
    const int b = slice_bits(k_block, slice_format);
    if (b < 0) return OZAKI_STATUS_INFEASIBLE;
    if (rho_out) *rho_out = 53 - b;
    if (bits_out) *bits_out = b;
    return 0;
}

int64_t ozaki_suggest_k_block(int64_t k, int slice_format) {
    if (k < 0) return -1;
    if (!format_ok(slice_format)) return -2;
    if (slice_format == OZAKI_SLICE_FP16) return k > 4096 ? 4096 : 0;
    if (slice_format == OZAKI_SLICE_INT8) return k > 524287 ? 262144 : 0;
    return k > 65536 ? MAX_K_BLOCK_IN_REGISTERS : 0;
}

int ozaki_set_stream(void* hip_stream) {
    ctx().stream = reinterpret_cast<hipStream_t>(hip_stream);
    return 0;
}

size_t ozaki_workspace_bytes_ex(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block, int pair_set,
                                int minimum) {
    Plan pl;
    if (plan_for_query(m, n, k, slice_format, num_slices, k_block, pair_set, pl) != 0) return 0;
    return minimum ? minimum_bytes(pl) : recommended_bytes(pl);
}

size_t ozaki_workspace_bytes(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block) {
    return ozaki_workspace_bytes_ex(m, n, k, slice_format, num_slices, k_block, OZAKI_PAIRS_TRIANGLE, 0);
}

size_t ozaki_workspace_min_bytes(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block) {
    return ozaki_workspace_bytes_ex(m, n, k, slice_format, num_slices, k_block, OZAKI_PAIRS_TRIANGLE, 1);
}

int ozaki_set_workspace(void* dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0)) return -1;
    if (reinterpret_cast<uintptr_t>(dev_ptr) % ALIGN != 0) return -1;
    if (dev_ptr && bytes < FLAG_BYTES) return -2;
    Context& c = ctx();
    c.ws = reinterpret_cast<uint8_t*>(dev_ptr);
    c.ws_bytes = bytes;
    if (c.ws) HIP_TRY(hipMemsetAsync(c.ws, 0, FLAG_BYTES, c.stream));
    return 0;
}

int ozaki_last_device_status(void) {
    // the flag words of the context's workspace and of this device's static scratch (if ozaki_dgemm_static has used it)
    Context& c = ctx();
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    uint8_t* places[2] = {c.ws, (dev >= 0 && dev < MAX_DEVICES) ? static_scratch_ptr[dev] : nullptr};
    int flags[2] = {0, 0};
    for (int i = 0; i < 2; ++i)
        if (places[i]) HIP_TRY(hipMemcpyAsync(&flags[i], places[i], sizeof(int), hipMemcpyDeviceToHost, c.stream));
    HIP_TRY(hipStreamSynchronize(c.stream));
    for (int i = 0; i < 2; ++i)
        if (flags[i]) HIP_TRY(hipMemsetAsync(places[i], 0, FLAG_BYTES, c.stream));
    return ((flags[0] | flags[1]) & 1) ? OZAKI_STATUS_NONFINITE : 0;
}

int ozaki_last_hip_error(void) { return ctx().last_hip_error; }

const char* ozaki_status_string(int status) {
    switch (status) {
        case OZAKI_STATUS_OK: return "success";
        case OZAKI_STATUS_INFEASIBLE: return "infeasible: no slice width keeps the matrix unit's accumulation exact for this block length";
        case OZAKI_STATUS_WORKSPACE: return "workspace missing or too small";
        case OZAKI_STATUS_HIP_ERROR: return "HIP runtime error";
        case OZAKI_STATUS_NONFINITE: return "non-finite input";
        case OZAKI_STATUS_STATIC_LIMIT: return "problem needs more work memory than the static scratch of ozaki_dgemm_static holds";
        case OZAKI_STATUS_SLICE_COUNT: return "num_slices exceeds OZAKI_MAX_SLICES";
        default: return status < 0 ? "invalid argument (the negated value is its 1-based position)" : "unknown status";
    }
}

int ozaki_profile_enable(int on) {
    ctx().profiling = on != 0;
    return 0;
}

int ozaki_profile_read(float* ms_out, int* launches_out) {
    if (!ms_out) return -1;
    Context& c = ctx();
    for (int i = 0; i < 3; ++i) { ms_out[i] = 0.0f; if (launches_out) launches_out[i] = 0; }
    // whatever happens below, every span leaves the list and its events return to the pool exactly once
    std::vector<Context::Span> spans;
    spans.swap(c.spans);
    hipError_t err = hipStreamSynchronize(c.stream);
    for (auto& sp : spans) {
        float ms = 0.0f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, sp.e0, sp.e1);
        if (err == hipSuccess) {
            ms_out[sp.phase] += ms;
            if (launches_out) launches_out[sp.phase] += 1;
        }
        c.pool.push_back(sp.e0);
        c.pool.push_back(sp.e1);
    }
    return err == hipSuccess ? 0 : fail_hip(err);
}

int ozaki_dgemm_ex(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb, double* C,
                   int64_t ldc, int slice_format, int num_slices, int64_t k_block, int accum_mode, int pair_set, int sum_rule,
                   size_t mem_cap) {
    const Options o{slice_format, num_slices, k_block, accum_mode, pair_set, sum_rule};
    Plan pl;
    const int st = check_dgemm_args(m, n, k, A, lda, B, ldb, C, ldc, o, pl);
    if (st != 0) return st;
    WorkMem wm = context_workspace();
    if (mem_cap == 0 || m == 0 || n == 0 || k == 0) return dgemm_core(pl, 1.0, A, lda, B, ldb, 0.0, C, ldc, o, wm);
    if (wm.bytes > mem_cap) wm.bytes = mem_cap;
    return dgemm_panels(pl, A, lda, B, ldb, C, ldc, o, wm);
}

int ozaki_dgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                double* C, int64_t ldc, int slice_format, int num_slices, int64_t k_block, int accum_mode) {
    return ozaki_dgemm_ex(m, n, k, A, lda, B, ldb, C, ldc, slice_format, num_slices, k_block, accum_mode, OZAKI_PAIRS_TRIANGLE,
                          OZAKI_SUM_RUNS, 0);
}

int ozaki_dgemm_static(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                       double* C, int64_t ldc, int slice_format, int num_slices, int64_t k_block, int accum_mode) {
    const Options o{slice_format, num_slices, k_block, accum_mode, OZAKI_PAIRS_TRIANGLE, OZAKI_SUM_RUNS};
    Plan pl;
    const int st = check_dgemm_args(m, n, k, A, lda, B, ldb, C, ldc, o, pl);
    if (st != 0) return st;
    if (m > 0 && n > 0 && k > 0 && minimum_bytes(pl) > (size_t)OZAKI_STATIC_SCRATCH_BYTES) return OZAKI_STATUS_STATIC_LIMIT;
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail_hip(hipErrorInvalidDevice);
    if (!static_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
        if (!p) return fail_hip(hipErrorInvalidSymbol);
        static_scratch_ptr[dev] = static_cast<uint8_t*>(p);
    }
    // Nothing in the scratch has to start at zero except the flag word, which is zero when the code object is loaded
    // and is cleared by ozaki_last_device_status after it has reported a flag: every other buffer of the carve-up is
    // written in full by the slicing and GEMM kernels before it is read.
    return dgemm_core(pl, 1.0, A, lda, B, ldb, 0.0, C, ldc, o, WorkMem{static_scratch_ptr[dev], (size_t)OZAKI_STATIC_SCRATCH_BYTES});
}

int ozaki_dgemm_scaled(int64_t m, int64_t n, int64_t k, double alpha, const double* A, int64_t lda, const double* B, int64_t ldb,
                       double beta, double* C, int64_t ldc, int slice_format, int num_slices, int64_t k_block, int accum_mode) {
    if (!scalar_ok(alpha)) return -4;
    if (!scalar_ok(beta)) return -9;
    const Options o{slice_format, num_slices, k_block, accum_mode, OZAKI_PAIRS_TRIANGLE, OZAKI_SUM_RUNS};
    Plan pl;
    int st = check_dgemm_args(m, n, k, A, lda, B, ldb, C, ldc, o, pl);
    if (st == 0) st = dgemm_core(pl, alpha, A, lda, B, ldb, beta, C, ldc, o, context_workspace());
    // argument positions of ozaki_dgemm -> positions in this signature (alpha and beta inserted)
    if (st < 0) return st >= -3 ? st : st >= -7 ? st - 1 : st - 2;
    return st;
}

size_t ozaki_workspace_bytes_scaled(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block) {
    Plan pl;
    if (make_plan(m, n, k, slice_format, num_slices, k_block, false, pl) != 0) return 0;
    return recommended_bytes(pl) + product_bytes(pl);
}

int ozaki_split(int is_B, int64_t rows, int64_t k, const double* X, int64_t ldx, int slice_format, int num_slices,
                int64_t k_block, void* slices_out, int32_t* exps_out) {
    if (is_B != 0 && is_B != 1) return -1;
    if (rows < 0) return -2;
    if (k < 0) return -3;
    if (num_slices < 1) return -7;
    Plan pl;
    // plan with the operand in the role it has in the product; the other dimension is irrelevant here
    const int st = make_plan(is_B ? 0 : rows, is_B ? rows : 0, k, slice_format, num_slices, k_block, false, pl);
    if (st < 0) return st == -10 ? -6 : st == -12 ? -8 : st;
    if (st != 0) return st;
    if (rows == 0 || k == 0) return 0;
    if (!X) return -4;
    if (ldx < (is_B ? (k > 1 ? k : 1) : (rows > 1 ? rows : 1))) return -5;
    if (!slices_out) return -9;
    if (!exps_out) return -10;
    Carve c;
    if (!carve(pl, c, false, context_workspace())) return OZAKI_STATUS_WORKSPACE;
    int rc = run_split(pl, c, X, ldx, X, ldx, !is_B, is_B != 0);
    if (rc) return rc;
    hipStream_t stream = ctx().stream;
    const Operand& op = is_B ? c.B : c.A;
    HIP_TRY(launch_export_slices(pl, op, slices_out, stream));
    // exponents: [T][s][rows_pad] -> [T][s][rows]
    HIP_TRY(hipMemcpy2DAsync(exps_out, (size_t)rows * sizeof(int32_t), op.exps, (size_t)op.rows_pad * sizeof(int32_t),
                             (size_t)rows * sizeof(int32_t), (size_t)pl.T * pl.s, hipMemcpyDeviceToDevice, stream));
    return 0;
}

int ozaki_count_slices(int is_B, int64_t rows, int64_t k, const double* X, int64_t ldx, int slice_format, int64_t k_block,
                       int* count_out) {
    if (is_B != 0 && is_B != 1) return -1;
    if (rows < 0) return -2;
    if (k < 0) return -3;
    if (!count_out) return -8;
    Plan pl;
    const int st = make_plan(is_B ? 0 : rows, is_B ? rows : 0, k, slice_format, 1, k_block, false, pl);
    if (st < 0) return st == -10 ? -6 : st == -12 ? -7 : st;
    if (st != 0) return st;
    *count_out = 0;
    if (rows == 0 || k == 0) return 0;
    if (!X) return -4;
    if (ldx < (is_B ? (k > 1 ? k : 1) : (rows > 1 ? rows : 1))) return -5;
    // needs the flag block, for A room for its transpose, and for long blocks the streaming kernel's state
    Context& c = ctx();
    const size_t at_bytes = is_B ? 0 : align_up((size_t)rows * k * sizeof(double));
    const size_t need = FLAG_BYTES + at_bytes + state_bytes(pl);
    if (!c.ws || c.ws_bytes < need) return OZAKI_STATUS_WORKSPACE;
    int* flags = reinterpret_cast<int*>(c.ws);
    HIP_TRY(hipMemsetAsync(flags + 1, 0, sizeof(int), c.stream));
    const double* vecs = X;
    int64_t ldv = ldx;
    if (!is_B) {
        double* At = reinterpret_cast<double*>(c.ws + FLAG_BYTES);
        HIP_TRY(launch_transpose(X, ldx, rows, k, At, c.stream));
        vecs = At;
        ldv = k;
    }
    void* state = state_bytes(pl) ? c.ws + FLAG_BYTES + at_bytes : nullptr;
    HIP_TRY(launch_count_slices(vecs, ldv, pl, rows, flags, state, c.stream));
    int count = 0;
    HIP_TRY(hipMemcpyAsync(&count, flags + 1, sizeof(int), hipMemcpyDeviceToHost, c.stream));
    HIP_TRY(hipStreamSynchronize(c.stream));
    *count_out = count;
    return 0;
}

int ozaki_pair_products(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                        int slice_format, int num_slices, int64_t k_block, int pair_set, int chained, void* P_out,
                        uint8_t* run_len_out) {
    if (pair_set != OZAKI_PAIRS_TRIANGLE && pair_set != OZAKI_PAIRS_ALL) return -11;
    Plan pl;
    int st = make_plan(m, n, k, slice_format, num_slices, k_block, pair_set == OZAKI_PAIRS_ALL, pl);
    if (st < 0) return st == -10 ? -8 : st == -11 ? -9 : st == -12 ? -10 : st;
    if (st != 0) return st;
    if (num_slices < 1) return -9;
    if (m == 0 || n == 0 || k == 0) return 0;
    if (!A) return -4;
    if (lda < m) return -5;
    if (!B) return -6;
    if (ldb < k) return -7;
    if (!P_out) return -13;
    Carve c;
    if (!carve(pl, c, false, context_workspace())) return OZAKI_STATUS_WORKSPACE;
    hipStream_t stream = ctx().stream;
    const PairOrder order = order_of(pl);
    int rc = run_split(pl, c, A, lda, B, ldb, true, true);
    if (rc) return rc;
    for (int64_t t = 0; t < pl.T; ++t) {
        int z0 = 0;
        for (int g_hi = order_top_diag(order); g_hi >= 2;) {
            const Pass ps = next_pass(order, g_hi, c.chunk_pairs);
            const size_t at = ((size_t)t * pl.npairs + z0) * (size_t)m * n;
            HIP_TRY(launch_pair_gemm(pl, c.A, c.B, order, ps, chained != 0, t, c.P, stream));
            HIP_TRY(launch_export_products(pl, c.A, c.B, order, ps, chained != 0, t, c.P, static_cast<float*>(P_out) + at,
                                           run_len_out ? run_len_out + at : nullptr, stream));
            z0 += ps.npairs;
            g_hi = ps.g_lo - 1;
        }
    }
    return 0;
}

int ozaki_fp64_add_emulated(const double* a, const double* b, double* out, int64_t n) {
    if (n < 0) return -4;
    if (n == 0) return 0;
    if (!a) return -1;
    if (!b) return -2;
    if (!out) return -3;
    HIP_TRY(launch_add_emulated(a, b, out, n, ctx().stream));
    return 0;
}

}  // extern "C"
