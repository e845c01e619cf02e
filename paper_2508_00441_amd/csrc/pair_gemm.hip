// Slice-pair GEMMs on the gfx950 matrix unit (paper Section 3, Eq. 10-11; Section 4.1).
//
// For one k-block and one slice pair (p, q) the product  P[i][j] = sum_kk sliceA_p[i][kk] * sliceB_q[j][kk]
// is formed with FP8 (v_mfma_f32_32x32x64_f8f6f4) or FP16 (v_mfma_f32_32x32x16_f16) inputs and FP32
// accumulation.  Every slice entry is q*2^-b with |q| <= 2^b and k_block*4^b <= 2^24, so every partial sum
// is an integer multiple of 2^-2b below 2^(24-2b) in magnitude and the FP32 accumulation is exact (Eq. 11).
// Because the sum is exact, the order in which the inner index is consumed is irrelevant; the kernel
// feeds both operands with the same (arbitrary but identical) assignment of inner indices to lanes.
//
// Work decomposition: one workgroup of four waves (one per SIMD) computes a 256 x 256 block of P for one
// pair; each wave owns 128 x 128 (4 x 4 MFMA tiles of 32 x 32, 256 accumulator registers per lane).  The
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
#include <type_traits>

#include "layout.hpp"

namespace ozaki {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

struct GemmArgs {
    const uint8_t* sa;       // A slices of the block: [s][chunks][rows_pad_a][CHUNK_BYTES]
    const uint8_t* sb;       // B slices of the block
    float* P;                // [nz][tiles_n][tiles_m][TILE_ELEMS]
    int64_t rows_pad_a, rows_pad_b;
    int64_t chunks;
    int tiles_m, tiles_n;
    int z0;
    PairList pairs;
};

constexpr int BK = CHUNK_BYTES;                       // bytes of the inner dimension per row and stage
constexpr int NSTAGE = 4;
constexpr int STAGE_BYTES = 2 * TILE * BK;            // X tile + Y tile
constexpr int LPW = TILE * BK / 1024 / 4;             // direct-to-LDS load instructions per wave, operand and stage
static_assert(BK == 64, "the swizzle and the fragment addressing below assume 64-byte LDS rows");

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

template <bool FP16>
__global__ void __launch_bounds__(256) pair_gemm_kernel(const GemmArgs a) {
    constexpr int KS = FP16 ? 2 : 1;                  // MFMA k-steps per stage (32 resp. 64 bytes of k each)
    constexpr int READS = FP16 ? 8 : 16;              // 128-bit LDS reads per wave and k-step
    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave >> 1, wm = wave & 1;

    const int tiles = a.tiles_m * a.tiles_n;
    const int zl = blockIdx.x / tiles;
    const int tile = blockIdx.x - zl * tiles;
    const int tn = tile / a.tiles_m, tm = tile - tn * a.tiles_m;
    const int p = a.pairs.p[a.z0 + zl] - 1, q = a.pairs.q[a.z0 + zl] - 1;
    const int chunks = (int)a.chunks;

    // loader: a wave instruction fills 16 consecutive LDS rows; lane -> row lane/4, physical piece lane%4,
    // which must hold logical piece (lane%4) ^ ((row>>2)&3); the row group starts at a multiple of 16 rows.
    const unsigned lrow = lane >> 2, lpc = lane & 3;
    const unsigned goff = lrow * BK + ((lpc ^ ((lrow >> 2) & 3)) << 4);
    const size_t cs_x = (size_t)a.rows_pad_b * BK, cs_y = (size_t)a.rows_pad_a * BK;
    const uint8_t* xptr = a.sb + (size_t)q * chunks * cs_x + (size_t)tn * TILE * BK + (size_t)wave * LPW * 1024 + goff;
    const uint8_t* yptr = a.sa + (size_t)p * chunks * cs_y + (size_t)tm * TILE * BK + (size_t)wave * LPW * 1024 + goff;

    // fragments: lane reads row lane%32 of each 32-row MFMA tile; lane/32 selects the k-group
    const int frow = lane & 31, fg = lane >> 5;
    const int fsw = (frow >> 2) & 3;
    const int xbase = (wn * 128 + frow) * BK;
    const int ybase = TILE * BK + (wm * 128 + frow) * BK;

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Fetch the stage xptr/yptr point at into ring buffer `buf`; `advance` moves on to the next chunk.  In the
    // tail the pointers stay on the last chunk: the (unused) reload keeps the outstanding-load count uniform.
    auto issue_to = [&](int buf, bool advance) {
        uint8_t* lb = lds + buf * STAGE_BYTES + wave * LPW * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds(OZAKI_GPTR(xptr + i * 1024), OZAKI_LPTR(lb + i * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds(OZAKI_GPTR(yptr + i * 1024), OZAKI_LPTR(lb + TILE * BK + i * 1024), 16, 0, 0);
        if (advance) {
            xptr += cs_x;
            yptr += cs_y;
        }
    };

    typedef typename std::conditional<FP16, v8h, v8i>::type frag_t;
    frag_t xf[2][4], yf[2][4];
    auto read_frags = [&](int kc, int ks, int fb) {
        const uint8_t* base = lds + (kc % NSTAGE) * STAGE_BYTES;
        if constexpr (FP16) {
            const int c0 = ((2 * ks + fg) ^ fsw) << 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) xf[fb][i] = *reinterpret_cast<const v8h*>(base + xbase + i * 32 * BK + c0);
#pragma unroll
            for (int j = 0; j < 4; ++j) yf[fb][j] = *reinterpret_cast<const v8h*>(base + ybase + j * 32 * BK + c0);
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
            for (int j = 0; j < 4; ++j) {
                if constexpr (FP16) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf[fb][i], yf[fb][j], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xf[fb][i], yf[fb][j], acc[i][j], 0, 0, 0, 0, 0, 0);
            }
    };

    // prologue: fill the ring, wait for stage 0, read its first fragments
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s) issue_to(s, s + 1 < chunks);
    wait_and_barrier<(NSTAGE - 1) * 2 * LPW>();
    read_frags(0, 0, 0);

    // One k-step: fetch the fragments of the next k-step into the other register buffer, then 16 MFMAs on the
    // current one.  At the last k-step of a stage: every wave waits for its own LDS reads and for the next
    // stage's loads, all waves meet, the next stage's first fragments are read and the dead buffer is refilled.
    auto kstep = [&](int g, auto fbc) {
        constexpr int fb = decltype(fbc)::value;
        const int kc = g / KS, ks = g % KS;
        const bool last_of_stage = ks + 1 == KS;
        if (!last_of_stage) {
            read_frags(kc, ks + 1, fb ^ 1);
        } else {
            wait_and_barrier<(NSTAGE - 2) * 2 * LPW>();
            read_frags(kc + 1 < chunks ? kc + 1 : kc, 0, fb ^ 1);
            issue_to(kc % NSTAGE, kc + NSTAGE + 1 < chunks);
        }
        mfmas(fb);
        // instruction order: the LDS reads behind the first MFMAs (so their latency is covered by the rest of
        // the k-step), the direct-to-LDS loads behind the later ones
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    // one MFMA
            if (i < 8) __builtin_amdgcn_sched_group_barrier(0x100, READS / 8, 0);                 // LDS reads
            else if (last_of_stage) __builtin_amdgcn_sched_group_barrier(0x020, 2 * LPW / 8, 0);  // VMEM reads
        }
    };
    const int ksteps = chunks * KS;
    int g = 0;
    for (; g + 1 < ksteps; g += 2) {
        kstep(g, std::integral_constant<int, 0>());
        kstep(g + 1, std::integral_constant<int, 1>());
    }
    if (g < ksteps) kstep(g, std::integral_constant<int, 0>());

    // every direct-to-LDS load (including the tail's unused reloads) must have landed before the workgroup's
    // LDS allocation is released
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");

    float* out = a.P + ((size_t)(zl * a.tiles_n + tn) * a.tiles_m + tm) * TILE_ELEMS + (size_t)wave * 16384 + lane * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                v4f v = {acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]};
                *reinterpret_cast<v4f*>(out + ((i * 4 + j) * 4 + g4) * 256) = v;
            }
}

}  // namespace

hipError_t launch_pair_gemm(const Plan& pl, const Operand& A, const Operand& B, const PairList& pairs,
                            int64_t t, int z0, int nz, float* P, hipStream_t st) {
    if (nz <= 0 || pl.tiles_m == 0 || pl.tiles_n == 0 || pl.chunks == 0) return hipSuccess;
    GemmArgs a;
    const size_t slice_a = (size_t)pl.chunks * A.rows_pad * CHUNK_BYTES, slice_b = (size_t)pl.chunks * B.rows_pad * CHUNK_BYTES;
    a.sa = A.slices + (size_t)t * pl.s * slice_a;
    a.sb = B.slices + (size_t)t * pl.s * slice_b;
    a.P = P;
    a.rows_pad_a = A.rows_pad; a.rows_pad_b = B.rows_pad; a.chunks = pl.chunks;
    a.tiles_m = (int)pl.tiles_m; a.tiles_n = (int)pl.tiles_n; a.z0 = z0; a.pairs = pairs;
    const int64_t blocks = (int64_t)nz * pl.tiles_m * pl.tiles_n;
    if (blocks > 0x7FFFFFFF || pl.chunks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (pl.fmt == 1) hipLaunchKernelGGL((pair_gemm_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((pair_gemm_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ozaki
