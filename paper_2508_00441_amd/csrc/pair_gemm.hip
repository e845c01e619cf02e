// Slice-pair GEMMs on the gfx950 matrix unit (paper Section 3, Eq. 10-11; Section 4.1).
//
// For one k-block and one slice pair (p, q) the product  P[i][j] = sum_kk sliceA_p[i][kk] * sliceB_q[j][kk]
// is formed with FP8 (v_mfma_f32_32x32x64_f8f6f4) or FP16 (v_mfma_f32_32x32x16_f16) inputs and FP32
// accumulation.  Every slice entry is q*2^-b with |q| <= 2^b and k_block*4^b <= 2^24, so every partial sum
// is an integer multiple of 2^-2b below 2^(24-2b) in magnitude and the FP32 accumulation is exact (Eq. 11).
// Because the sum is exact, the order in which the inner index is consumed is irrelevant; the kernel
// feeds both operands with the same (arbitrary but identical) assignment of inner indices to lanes.
//
// Work decomposition: one workgroup of four waves computes a 256 x 256 block of P for one pair; each wave
// owns 128 x 128 (4 x 4 MFMA tiles of 32 x 32, 256 accumulator registers per lane).  The matrix unit's
// "row" operand is the B slice (index n), its "column" operand the A slice (index m), so that the lanes
// of a wave run along m, the contiguous direction of column-major C.
// Per step, 128 bytes of the inner dimension of 256 + 256 slice vectors (2 x 32 KiB, contiguous in the
// slice layout) are staged through LDS, double buffered.  LDS rows are 128 bytes; the 16-byte pieces of a
// row are XOR-swizzled with bits 1..3 of the row number so that the 16 lanes served together by a
// 128-bit LDS read hit 64 distinct banks.
#include "layout.hpp"

namespace ozaki {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

struct GemmArgs {
    const uint8_t* sa;       // A slices of the block: [s][chunks][rows_pad_a][128]
    const uint8_t* sb;       // B slices of the block
    float* P;                // [nz][tiles_n][tiles_m][TILE_ELEMS]
    int64_t rows_pad_a, rows_pad_b;
    int64_t chunks;
    int tiles_m, tiles_n;
    int z0;
    PairList pairs;
};

constexpr int STAGE_BYTES = 2 * TILE * CHUNK_BYTES;     // X tile + Y tile

template <bool FP16>
__global__ void __launch_bounds__(256) pair_gemm_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wn = wave >> 1, wm = wave & 1;

    const int tiles = a.tiles_m * a.tiles_n;
    const int zl = blockIdx.x / tiles;
    const int tile = blockIdx.x - zl * tiles;
    const int tn = tile / a.tiles_m, tm = tile - tn * a.tiles_m;
    const int p = a.pairs.p[a.z0 + zl] - 1, q = a.pairs.q[a.z0 + zl] - 1;

    const size_t chunk_stride_x = (size_t)a.rows_pad_b * CHUNK_BYTES;
    const size_t chunk_stride_y = (size_t)a.rows_pad_a * CHUNK_BYTES;
    const uint8_t* xg = a.sb + (size_t)q * a.chunks * chunk_stride_x + (size_t)tn * TILE * CHUNK_BYTES + tid * 16;
    const uint8_t* yg = a.sa + (size_t)p * a.chunks * chunk_stride_y + (size_t)tm * TILE * CHUNK_BYTES + tid * 16;

    // staging: thread tid moves bytes [tid*16 + i*4096, +16) of each 32 KiB tile, i = 0..7: row tid/8 + 32 i, piece tid%8
    const int wrow = tid >> 3;
    const int waddr = wrow * CHUNK_BYTES + (((tid & 7) ^ ((wrow >> 1) & 7)) << 4);

    // fragments: lane reads row (lane%32) of each 32-row MFMA tile, 16-byte pieces chosen by lane/32 and the k-step
    const int frow = lane & 31, fg = lane >> 5;
    const int fsw = (frow >> 1) & 7;
    const int xbase = (wn * 128 + frow) * CHUNK_BYTES;
    const int ybase = TILE * CHUNK_BYTES + (wm * 128 + frow) * CHUNK_BYTES;

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    v4i stx[8], sty[8];
    auto gload = [&](int64_t kc) {
        const uint8_t* xs = xg + kc * chunk_stride_x;
        const uint8_t* ys = yg + kc * chunk_stride_y;
#pragma unroll
        for (int i = 0; i < 8; ++i) stx[i] = *reinterpret_cast<const v4i*>(xs + i * 4096);
#pragma unroll
        for (int i = 0; i < 8; ++i) sty[i] = *reinterpret_cast<const v4i*>(ys + i * 4096);
    };
    auto lstore = [&](int buf) {
        uint8_t* base = lds + buf * STAGE_BYTES + waddr;
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<v4i*>(base + i * 4096) = stx[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<v4i*>(base + TILE * CHUNK_BYTES + i * 4096) = sty[i];
    };
    auto compute = [&](int buf) {
        const uint8_t* base = lds + buf * STAGE_BYTES;
        if constexpr (!FP16) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int c0 = ((4 * ks + 2 * fg) ^ fsw) << 4, c1 = ((4 * ks + 2 * fg + 1) ^ fsw) << 4;
                v8i xf[4], yf[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const v4i lo = *reinterpret_cast<const v4i*>(base + xbase + i * 32 * CHUNK_BYTES + c0);
                    const v4i hi = *reinterpret_cast<const v4i*>(base + xbase + i * 32 * CHUNK_BYTES + c1);
                    xf[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const v4i lo = *reinterpret_cast<const v4i*>(base + ybase + j * 32 * CHUNK_BYTES + c0);
                    const v4i hi = *reinterpret_cast<const v4i*>(base + ybase + j * 32 * CHUNK_BYTES + c1);
                    yf[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xf[i], yf[j], acc[i][j], 0, 0, 0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int c0 = ((2 * ks + fg) ^ fsw) << 4;
                v8h xf[4], yf[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) xf[i] = *reinterpret_cast<const v8h*>(base + xbase + i * 32 * CHUNK_BYTES + c0);
#pragma unroll
                for (int j = 0; j < 4; ++j) yf[j] = *reinterpret_cast<const v8h*>(base + ybase + j * 32 * CHUNK_BYTES + c0);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf[i], yf[j], acc[i][j], 0, 0, 0);
            }
        }
    };

    gload(0);
    lstore(0);
    __syncthreads();
    for (int64_t kc = 0; kc < a.chunks; ++kc) {
        const bool more = kc + 1 < a.chunks;
        if (more) gload(kc + 1);
        compute((int)(kc & 1));
        if (more) lstore((int)((kc + 1) & 1));
        __syncthreads();
    }

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
    if (nz <= 0 || pl.tiles_m == 0 || pl.tiles_n == 0) return hipSuccess;
    GemmArgs a;
    const size_t slice_a = (size_t)pl.chunks * A.rows_pad * CHUNK_BYTES, slice_b = (size_t)pl.chunks * B.rows_pad * CHUNK_BYTES;
    a.sa = A.slices + (size_t)t * pl.s * slice_a;
    a.sb = B.slices + (size_t)t * pl.s * slice_b;
    a.P = P;
    a.rows_pad_a = A.rows_pad; a.rows_pad_b = B.rows_pad; a.chunks = pl.chunks;
    a.tiles_m = (int)pl.tiles_m; a.tiles_n = (int)pl.tiles_n; a.z0 = z0; a.pairs = pairs;
    const int64_t blocks = (int64_t)nz * pl.tiles_m * pl.tiles_n;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (pl.fmt == 1) hipLaunchKernelGGL((pair_gemm_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((pair_gemm_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ozaki
