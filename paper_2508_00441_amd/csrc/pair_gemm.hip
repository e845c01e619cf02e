// Slice-pair GEMMs on the gfx950 matrix unit (paper Section 3, Eq. 10-11; Section 4.1).
//
// For one k-block and one slice pair (p, q) the product  P[i][j] = sum_kk sliceA_p[i][kk] * sliceB_q[j][kk]
// is formed with FP8 or FP6 (v_mfma_f32_32x32x64_f8f6f4; FP6 codes hold twice the slice value, which the
// accumulation kernel undoes with the exponents) or FP16 (v_mfma_f32_32x32x16_f16) inputs and FP32
// accumulation, or with INT8 inputs and INT32 accumulation (v_mfma_i32_32x32x32_i8; the slice entries are then the
// integers q themselves and the sums are exact up to 2^31 - 1).  Every slice entry is q*2^-b with |q| <= 2^b and k_block*4^b <= 2^24, so every partial sum
// is an integer multiple of 2^-2b below 2^(24-2b) in magnitude and the FP32 accumulation is exact (Eq. 11).
// Because the sum is exact, the order in which the inner index is consumed is irrelevant; the kernel
// feeds both operands with the same (arbitrary but identical) assignment of inner indices to lanes.
//
// Work decomposition: one workgroup of four waves (one per SIMD) computes a 256 x 256 block of P for one
// group of pairs (consecutive pairs of an anti-diagonal, streamed through one continuous pipeline); each wave owns
// 128 x 128 (4 x 4 MFMA tiles of 32 x 32, 256 accumulator registers per lane).  Whether the product of the next pair
// keeps accumulating on top of the current one is decided per 32 x 32 MFMA tile: it does where all 32 rows of A and all
// 32 columns of B concerned carry the same scale factor for both pairs (exact, because a group never exceeds the
// window of Eq. 11); a tile that does not is stored and cleared, so one irregular row costs one 4 KiB store, not the
// workgroup's 256 KiB.  The
// matrix unit's "row" operand is the B slice (index n), its "column" operand the A slice (index m), so that
// the lanes of a wave run along m, the contiguous direction of column-major C.
//
// Pipeline: a stage is 64 bytes of the inner dimension of 256 + 256 slice vectors (2 x 16 KiB, each
// contiguous in the slice layout).  Stages travel HBM/L2 -> LDS with direct-to-LDS loads
// (global_load_lds_dwordx4) through a ring of NSTAGE buffers; fragments travel LDS -> registers one k-step
// ahead of the MFMAs that consume them (register double buffering).  Once a wave holds the fragments of a
// stage's last k-step in registers the stage buffer is dead, so the buffer is refilled right after the
// barrier that also publishes the next stage.  Inside a k-step the LDS reads and the direct-to-LDS loads are
// spread between the 16 MFMAs (sched_group_barrier), which keeps the LDS command queue short and the matrix
// pipe fed by a single wave per SIMD.
//
// LDS rows are 64 bytes; the four 16-byte pieces of a row are XOR-swizzled with bits 2..3 of the row number
// so that the 16 lanes served together by a 128-bit LDS read hit 64 distinct banks.  A direct-to-LDS load
// writes lane L's 16 bytes at (wave-uniform base) + 16 L, so the swizzle is applied on the global side: each
// lane fetches the piece that belongs at its fixed LDS position.
//
// FP6 stages are 48 bytes per vector, kept in the four planes of the slice layout ([k-group][vector][16 B] and
// [k-group][vector][8 B]): every plane of a tile is contiguous in memory, is copied as it is, and a wave's fragment
// reads (one 128-bit and one 64-bit read per 32 x 64 operand tile) are contiguous, so no swizzle is needed.
#include <type_traits>

#include "layout.hpp"

namespace ozaki {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

struct GemmArgs {
    const uint8_t* sa;       // A slices of the block: [s][chunks][rows_pad_a][row bytes]
    const uint8_t* sb;       // B slices of the block
    float* P;                // [nz][tiles_n][tiles_m][TILE_ELEMS]
    int64_t rows_pad_a, rows_pad_b;
    int64_t chunks;
    int tiles_m, tiles_n;
    int allow_chain;
    const int32_t* da;       // A deltas of the block: [s][rows_pad_a / 32]
    const int32_t* db;       // B deltas of the block: [s][rows_pad_b / 32]
    PairOrder order;
    Pass pass;
};

static_assert(CHUNK_BYTES == 64, "the swizzle and the fragment addressing below assume 64-byte LDS rows");

#define OZAKI_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define OZAKI_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// Wait until at most N vector-memory operations of this wave are outstanding and all its LDS operations have
// completed, then meet the other waves.  No memory fence is attached (a fence would force vmcnt(0) and
// serialise the pipeline); the empty asm statements keep the compiler from moving memory operations across.
template <int N>
__device__ __forceinline__ void wait_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0070);   // vmcnt(N) expcnt(7) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int FMT>
__global__ void __launch_bounds__(256) pair_gemm_kernel(const GemmArgs a) {
    constexpr bool FP16 = FMT == FMT_FP16;
    constexpr bool INT8 = FMT == FMT_INT8;
    constexpr bool HALF = FP16 || INT8;               // 16-byte fragments, two k-steps per 64-byte stage
    constexpr bool FP6 = fmt_is_fp6(FMT);
    constexpr int FP6_CODE = FMT == FMT_FP6_E3M2 ? 3 : 2;     // operand format field of the instruction: 2 = E2M3, 3 = E3M2
    constexpr int BK = FP6 ? CHUNK_BYTES_FP6 : CHUNK_BYTES;   // bytes of the inner dimension per vector and stage
    constexpr int OPERAND_BYTES = TILE * BK;          // one operand's share of a stage
    constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;    // X tile + Y tile
    constexpr int LPW = OPERAND_BYTES / 1024 / 4;     // direct-to-LDS load instructions per wave, operand and stage
    constexpr int NSTAGE = FP6 ? 6 : 5;               // ring of stage buffers: 5 x 32 KiB resp. 6 x 24 KiB of the 160 KiB LDS
    constexpr int KS = HALF ? 2 : 1;                  // MFMA k-steps per stage (half a stage's bytes, or all of them, each)
    constexpr int READS = HALF ? 8 : 16;              // LDS read instructions per wave and k-step
    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave >> 1, wm = wave & 1;

    // one workgroup = one tile of one group of pairs (p0 + j, q0 - j), j < glen
    const int tiles = a.tiles_m * a.tiles_n;
    const int gi = blockIdx.x / tiles;
    const int tile = blockIdx.x - gi * tiles;
    const int tn = tile / a.tiles_m, tm = tile - tn * a.tiles_m;
    const Group grp = pass_group(a.order, a.pass, gi);
    const int glen = grp.len, p0 = grp.p0 - 1, q0 = grp.q0 - 1;       // 0-based slice indices from here on
    const int chunks = (int)a.chunks;
    // Whether pair jp+1 of the group keeps accumulating on top of pair jp is decided per MFMA tile (i, j) of the wave,
    // when pair jp is complete: it does if all 32 rows of A and all 32 columns of B behind the tile carry the same scale
    // factor for both pairs (pair_linked; the sum stays inside the exact window because a group has at most run_limit
    // pairs).  The rows of A behind tile column j are the 32-vector group tm*8 + wm*4 + j, the columns of B behind
    // tile row i the group tn*8 + wn*4 + i.  The deltas of the wave's four groups are 16 contiguous bytes per slice and
    // are read through the scalar cache (they were written by an earlier kernel and the addresses are wave-uniform), so
    // they stay out of the vector-memory counter that paces the load ring.
    typedef int v4s __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(4))) v4s* delta4_ptr;
    const int64_t groups_a = a.rows_pad_a / LINK_ROWS, groups_b = a.rows_pad_b / LINK_ROWS;
    // the four consecutive groups of this wave, for slice 0: 16 bytes, 16-byte aligned (slice p follows p * groups later)
    const int32_t* const dA = a.da + (tm * 8 + wm * 4);
    const int32_t* const dB = a.db + (tn * 8 + wn * 4);
    // bit i*4+j: tile (i, j) continues its run after pair jp (0-based position in the group)
    auto continue_mask = [&](int jp) -> unsigned {
        if (!a.allow_chain) return 0u;
        const v4s dav = *(delta4_ptr)(dA + (size_t)(p0 + jp) * groups_a);
        const v4s dbv = *(delta4_ptr)(dB + (size_t)(q0 - jp - 1) * groups_b);
        unsigned cont = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                cont |= deltas_link(__builtin_amdgcn_readfirstlane(dav[j]), __builtin_amdgcn_readfirstlane(dbv[i])) ? (1u << (i * 4 + j)) : 0u;
        return cont;
    };

    // loader.  FP8/FP16: a wave instruction fills 16 consecutive LDS rows; lane -> row lane/4, physical piece lane%4,
    // which must hold logical piece (lane%4) ^ ((row>>2)&3); the row group starts at a multiple of 16 rows; a wave's
    // LPW instructions cover consecutive kilobytes of the tile.  FP6: every instruction copies one kilobyte of one
    // plane as it is; wave w takes kilobyte w of either 16-byte plane (4 KiB per tile each) and kilobyte w of the two
    // 8-byte planes taken together (2 KiB per tile each).
    const size_t cs_x = (size_t)a.rows_pad_b * BK, cs_y = (size_t)a.rows_pad_a * BK;      // chunk strides
    const uint8_t* xtile;
    const uint8_t* ytile;
    size_t xpiece[LPW], ypiece[LPW];                  // byte offset of the wave's i-th instruction from xptr / yptr
    if constexpr (FP6) {
        xtile = a.sb + lane * 16;
        ytile = a.sa + lane * 16;
        const size_t rb = (size_t)a.rows_pad_b, ra = (size_t)a.rows_pad_a;
        xpiece[0] = (size_t)tn * TILE * 16 + wave * 1024;
        xpiece[1] = rb * 16 + xpiece[0];
        xpiece[2] = rb * 32 + (size_t)(wave >> 1) * rb * 8 + (size_t)tn * TILE * 8 + (wave & 1) * 1024;
        ypiece[0] = (size_t)tm * TILE * 16 + wave * 1024;
        ypiece[1] = ra * 16 + ypiece[0];
        ypiece[2] = ra * 32 + (size_t)(wave >> 1) * ra * 8 + (size_t)tm * TILE * 8 + (wave & 1) * 1024;
    } else {
        const unsigned lrow = lane >> 2, lpc = lane & 3;
        const unsigned goff = lrow * BK + ((lpc ^ ((lrow >> 2) & 3)) << 4);
        xtile = a.sb + (size_t)tn * TILE * BK + (size_t)wave * LPW * 1024 + goff;
        ytile = a.sa + (size_t)tm * TILE * BK + (size_t)wave * LPW * 1024 + goff;
#pragma unroll
        for (int i = 0; i < LPW; ++i) xpiece[i] = ypiece[i] = (size_t)i * 1024;
    }
    // where the wave's i-th instruction lands inside an operand's share of a stage
    auto lds_piece = [&](int i) -> int { return FP6 ? i * 4096 + wave * 1024 : (wave * LPW + i) * 1024; };
    const uint8_t* xptr;
    const uint8_t* yptr;

    // fragments: lane reads row lane%32 of each 32-row MFMA tile; lane/32 selects the k-group
    const int frow = lane & 31, fg = lane >> 5;
    const int fsw = (frow >> 2) & 3;
    const int xrow = wn * 128 + frow, yrow = wm * 128 + frow;
    const int xbase = xrow * BK;
    const int ybase = OPERAND_BYTES + yrow * BK;

    typedef typename std::conditional<INT8, v16i, v16f>::type acc_t;      // INT32 or FP32 accumulators
    typedef typename std::conditional<INT8, v4i, v4f>::type acc4_t;
    acc_t acc[4][4];
    auto zero_tile = [&](acc_t& t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) t[r] = 0;
    };
    // the wave's part of the product slot `slot`, MFMA tile (i, j): 4 KiB contiguous, 16 bytes per lane and quarter.
    // The tile's base address is wave-uniform (it stays in scalar registers), the lane adds a 32-bit byte offset.
    const unsigned lane_bytes = (unsigned)lane * 16u;
    auto store_tile = [&](int slot, int i, int j, const acc_t& t) {
        char* base = reinterpret_cast<char*>(a.P + ((size_t)(slot * a.tiles_n + tn) * a.tiles_m + tm) * TILE_ELEMS + (size_t)wave * 16384 +
                                             (size_t)(i * 4 + j) * 1024);
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            acc4_t v = {t[4 * g4], t[4 * g4 + 1], t[4 * g4 + 2], t[4 * g4 + 3]};
            *reinterpret_cast<acc4_t*>(base + g4 * 1024 + lane_bytes) = v;
        }
    };

    // The group's pairs are streamed as one sequence of glen * chunks stages.  The A slices p0, p0+1, ... lie back
    // to back in memory, so yptr simply moves one chunk per stage; the B slices run backwards (q0, q0-1, ...), so
    // xptr jumps back by two slices minus one chunk when a pair ends.  After the last stage the pointers stay put:
    // the (unused) reloads keep the outstanding-load count uniform.
    const int total = glen * chunks;
    int issued = 0, issue_kc = 0;
    xptr = xtile + (size_t)q0 * chunks * cs_x;
    yptr = ytile + (size_t)p0 * chunks * cs_y;
    const size_t x_wrap = (size_t)(2 * chunks - 1) * cs_x;
    auto issue_next = [&](int buf) {
        uint8_t* lb = lds + buf * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds(OZAKI_GPTR(xptr + xpiece[i]), OZAKI_LPTR(lb + lds_piece(i)), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds(OZAKI_GPTR(yptr + ypiece[i]), OZAKI_LPTR(lb + OPERAND_BYTES + lds_piece(i)), 16, 0, 0);
        // branch-free pointer update (a branch here would split the k-step's basic block and with it the
        // instruction interleaving)
        const bool adv = issued + 1 < total;
        const bool wrap = issue_kc + 1 == chunks;
        const int64_t dx = adv ? (wrap ? -(int64_t)x_wrap : (int64_t)cs_x) : 0;
        const int64_t dy = adv ? (int64_t)cs_y : 0;
        xptr += dx;
        yptr += dy;
        issued += adv ? 1 : 0;
        issue_kc = adv ? (wrap ? 0 : issue_kc + 1) : issue_kc;
    };

    typedef typename std::conditional<FP16, v8h, typename std::conditional<INT8, v4i, v8i>::type>::type frag_t;
    frag_t xf[2][4], yf[2][4];
    auto read_frags = [&](int stage, int ks, int fb) {
        const uint8_t* base = lds + ((unsigned)stage % NSTAGE) * STAGE_BYTES;
        if constexpr (HALF) {
            const int c0 = ((2 * ks + fg) ^ fsw) << 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) xf[fb][i] = *reinterpret_cast<const frag_t*>(base + xbase + i * 32 * BK + c0);
#pragma unroll
            for (int j = 0; j < 4; ++j) yf[fb][j] = *reinterpret_cast<const frag_t*>(base + ybase + j * 32 * BK + c0);
        } else if constexpr (FP6) {
            // 24 bytes per lane: 16 from the 16-byte plane of its k-group, 8 from the 8-byte plane; the last two
            // registers of the operand are not read by the instruction for 6-bit formats
            const uint8_t* x16 = base + fg * 4096 + xrow * 16;
            const uint8_t* y16 = base + OPERAND_BYTES + fg * 4096 + yrow * 16;
            const unsigned x8 = (unsigned)(uintptr_t)OZAKI_LPTR(base + 8192 + fg * 2048 + xrow * 8);
            const unsigned y8 = (unsigned)(uintptr_t)OZAKI_LPTR(base + OPERAND_BYTES + 8192 + fg * 2048 + yrow * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // every 64-bit read gets an address register of its own (the empty asm hides their common origin):
                // merged into two-address reads they would land in registers that belong to two different operands
                // and would have to be moved, with a wait for the LDS in the middle of the k-step
                unsigned ax = x8 + i * 32 * 8, ay = y8 + i * 32 * 8;
                asm volatile("" : "+v"(ax), "+v"(ay));
                const v4i xlo = *reinterpret_cast<const v4i*>(x16 + i * 32 * 16);
                const v2i xhi = *reinterpret_cast<const __attribute__((address_space(3))) v2i*>((uintptr_t)ax);
                xf[fb][i] = __builtin_shufflevector(xlo, __builtin_shufflevector(xhi, xhi, 0, 1, -1, -1), 0, 1, 2, 3, 4, 5, -1, -1);
                const v4i ylo = *reinterpret_cast<const v4i*>(y16 + i * 32 * 16);
                const v2i yhi = *reinterpret_cast<const __attribute__((address_space(3))) v2i*>((uintptr_t)ay);
                yf[fb][i] = __builtin_shufflevector(ylo, __builtin_shufflevector(yhi, yhi, 0, 1, -1, -1), 0, 1, 2, 3, 4, 5, -1, -1);
            }
        } else {
            const int c0 = ((2 * fg) ^ fsw) << 4, c1 = ((2 * fg + 1) ^ fsw) << 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const v4i lo = *reinterpret_cast<const v4i*>(base + xbase + i * 32 * BK + c0);
                const v4i hi = *reinterpret_cast<const v4i*>(base + xbase + i * 32 * BK + c1);
                xf[fb][i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v4i lo = *reinterpret_cast<const v4i*>(base + ybase + j * 32 * BK + c0);
                const v4i hi = *reinterpret_cast<const v4i*>(base + ybase + j * 32 * BK + c1);
                yf[fb][j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    auto mfmas = [&](int fb) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int j = (i & 1) ? 3 - jj : jj;      // boustrophedon: consecutive MFMAs differ in one operand only
                if constexpr (FP16) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf[fb][i], yf[fb][j], acc[i][j], 0, 0, 0);
                else if constexpr (INT8) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xf[fb][i], yf[fb][j], acc[i][j], 0, 0, 0);
                else if constexpr (FP6) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xf[fb][i], yf[fb][j], acc[i][j], FP6_CODE, FP6_CODE, 0, 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xf[fb][i], yf[fb][j], acc[i][j], 0, 0, 0, 0, 0, 0);
            }
    };

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) zero_tile(acc[i][j]);
    // prologue: fill the ring, wait for stage 0, read its first fragments
#pragma unroll
    for (int st = 0; st < NSTAGE; ++st) issue_next(st);
    wait_and_barrier<(NSTAGE - 1) * 2 * LPW>();
    read_frags(0, 0, 0);

    // One k-step: fetch the fragments of the next k-step into the other register buffer, then 16 MFMAs on the
    // current one.  At the last k-step of a stage: every wave waits for its own LDS reads and for the next
    // stage's loads, all waves meet, the next stage's first fragments are read and the dead buffer is refilled.
    int stage = 0;
    auto kstep = [&](auto fbc, auto ksc) {
        constexpr int fb = decltype(fbc)::value;
        constexpr int ks = decltype(ksc)::value;
        constexpr bool last_of_stage = ks + 1 == KS;
        if constexpr (!last_of_stage) {
            read_frags(stage, ks + 1, fb ^ 1);
        } else {
            wait_and_barrier<(NSTAGE - 2) * 2 * LPW>();
            read_frags(stage + 1 < total ? stage + 1 : stage, 0, fb ^ 1);
            issue_next((unsigned)stage % NSTAGE);
        }
        mfmas(fb);
        // instruction order: the LDS reads behind the first MFMAs (so their latency is covered by the rest of
        // the k-step), the direct-to-LDS loads behind the later ones
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    // one MFMA
            if (i < 8) __builtin_amdgcn_sched_group_barrier(0x100, READS / 8, 0);                 // LDS reads
            else if (last_of_stage && i - 8 < 2 * LPW) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // a VMEM read
        }
        if constexpr (last_of_stage) ++stage;
    };
    const std::integral_constant<int, 0> c0;
    const std::integral_constant<int, 1> c1;
    unsigned run_start[4] = {0u, 0u, 0u, 0u};           // byte j of word i: first pair of the run tile (i, j) is accumulating
    for (int jp = 0; jp < glen; ++jp) {
        // which tiles continue their run after this pair: the scalar loads behind this are issued now and have long
        // landed when the pair's last stage is done
        const bool last_pair = jp + 1 == glen;
        const unsigned cont = last_pair ? 0u : continue_mask(jp);
        if constexpr (KS == 1) {
            int c = 0;
            for (; c + 1 < chunks; c += 2) {
                kstep(c0, c0);
                kstep(c1, c0);
            }
            if (c < chunks) {
                kstep(c0, c0);
                // odd number of stages: the fragments just fetched for the next stage sit in buffer 1; the next
                // k-step reads buffer 0
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xf[0][i] = xf[1][i];
                    yf[0][i] = yf[1][i];
                }
            }
        } else {
            for (int c = 0; c < chunks; ++c) {
                kstep(c0, c0);
                kstep(c1, c1);
            }
        }
        // The pair is complete.  Every tile whose run the next pair does not continue is stored to the slot of the
        // run's first pair and cleared (the stores only make the next vmcnt wait stricter).
        if (cont != 0xFFFFu) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (!((cont >> (i * 4 + j)) & 1u)) {
                        store_tile(grp.slot + (int)((run_start[i] >> (8 * j)) & 0xFFu), i, j, acc[i][j]);
                        zero_tile(acc[i][j]);
                        run_start[i] = (run_start[i] & ~(0xFFu << (8 * j))) | ((unsigned)(jp + 1) << (8 * j));
                    }
        }
    }

    // every direct-to-LDS load of this wave (including the tail's unused reloads) must have landed before the
    // workgroup's LDS allocation is released
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
}

}  // namespace

hipError_t launch_pair_gemm(const Plan& pl, const Operand& A, const Operand& B, const PairOrder& order, const Pass& ps,
                            bool allow_chain, int64_t t, float* P, hipStream_t st) {
    if (ps.ngroups <= 0 || pl.tiles_m == 0 || pl.tiles_n == 0 || pl.chunks == 0) return hipSuccess;
    GemmArgs a;
    const size_t slice_a = (size_t)pl.chunks * A.rows_pad * pl.row_bytes, slice_b = (size_t)pl.chunks * B.rows_pad * pl.row_bytes;
    a.sa = A.slices + (size_t)t * pl.s * slice_a;
    a.sb = B.slices + (size_t)t * pl.s * slice_b;
    a.P = P;
    a.rows_pad_a = A.rows_pad; a.rows_pad_b = B.rows_pad; a.chunks = pl.chunks;
    a.tiles_m = (int)pl.tiles_m; a.tiles_n = (int)pl.tiles_n;
    a.allow_chain = allow_chain ? 1 : 0;
    a.da = A.deltas + (size_t)t * (A.rows_pad / LINK_ROWS) * pl.s;
    a.db = B.deltas + (size_t)t * (B.rows_pad / LINK_ROWS) * pl.s;
    a.order = order; a.pass = ps;
    const int64_t blocks = (int64_t)ps.ngroups * pl.tiles_m * pl.tiles_n;
    if (blocks > 0x7FFFFFFF || pl.chunks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (pl.fmt == FMT_FP16) hipLaunchKernelGGL((pair_gemm_kernel<FMT_FP16>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else if (pl.fmt == FMT_FP6) hipLaunchKernelGGL((pair_gemm_kernel<FMT_FP6>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else if (pl.fmt == FMT_FP6_E3M2) hipLaunchKernelGGL((pair_gemm_kernel<FMT_FP6_E3M2>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else if (pl.fmt == FMT_INT8) hipLaunchKernelGGL((pair_gemm_kernel<FMT_INT8>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((pair_gemm_kernel<FMT_FP8>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ozaki
