// Slicing of the FP64 operands into Type2 slices (paper Section 3, Eq. 4-8), integer arithmetic only.
//
// For a vector x (a row of A or a column of B restricted to one k-block) and p = 1..s:
//     c   = smallest integer with max|x^(p)| <= 2^c   (Eq. 4, evaluated exactly; 0 for a zero vector)
//     q_i = x^(p)_i / 2^(c-b) rounded to the nearest integer, ties to even       (Eq. 5-6)
//     x^(p+1)_i = x^(p)_i - q_i 2^(c-b)                                            (Eq. 7, exact)
//     slice^(p)_i = q_i 2^-b stored in Type2                                       (Eq. 8)
// Eq. 5-6 obtain q through (x + sigma) - sigma with sigma = 0.75 * 2^(rho+c) in FP64: x + sigma lies in the
// binade whose unit in the last place is 2^(rho+c-53) = 2^(c-b), sigma is an even multiple of that unit,
// so the FP64 addition rounds x to the nearest multiple of 2^(c-b) with ties to even q, and the
// subtraction of sigma is exact.  The kernel computes the same q with integers: once an element is within
// reach of the current unit it is kept as the signed 64-bit fixed-point number x^(p) / 2^(c-b) with 60-b
// fraction bits, which holds the element and every later remainder exactly (|x^(p)| <= 2^c bounds it by 2^60);
// q is its rounding to an integer, the remainder is what is left, and moving to the next slice is a left shift
// by c_p - c_(p+1).  Until then the element waits with its significand and exponent: with b <= 7 it is then smaller
// than half the unit (q = 0); with wider slices it can already reach the unit, and is rounded in its integer form.
// No FP64 instruction is executed.  Two forms of this element step: slices of at most 7 bits (FP8, FP6, INT8) work on
// the upper 32-bit word of the fixed-point number (slice_element.hpp); FP16 slices, whose fixed-point form has fewer
// than 53 fraction bits, keep the 64-bit step below (decode_element, slice_element).
//
// A vector is held in the registers of TPR threads (8*U consecutive elements per thread in U groups of
// eight) for all s slices, so HBM sees each input element once and each slice code once.
#include <string.h>

#include "layout.hpp"
#include "slice_element.hpp"

namespace ozaki {

namespace {

__global__ void __launch_bounds__(256) transpose_kernel(const double* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                        double* __restrict__ At) {
    __shared__ double tile[32][33];
    const int64_t i0 = (int64_t)blockIdx.x * 32, k0 = (int64_t)blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int j = ty; j < 32; j += 8) {
        int64_t i = i0 + tx, kk = k0 + j;
        if (i < m && kk < k) tile[j][tx] = A[i + kk * lda];
    }
    __syncthreads();
    for (int j = ty; j < 32; j += 8) {
        int64_t i = i0 + j, kk = k0 + tx;
        if (i < m && kk < k) At[i * k + kk] = tile[tx][j];
    }
}

// One operand of a split launch.
struct SplitVectors {
    const double* X;       // vector r starts at X + r*ldv
    int64_t ldv;
    int64_t rows, rows_pad;
    int vec_ok;            // 16-byte aligned loads allowed
    uint8_t* slices;       // null: count only, nothing is stored
    int32_t* exps;
};

// A launch splits the vectors of up to two operands (same k, block length, format and slice count): the first wg_first
// workgroups of the grid belong to v[0], the rest to v[1].
struct SplitArgs {
    SplitVectors v[2];
    unsigned wg_first;     // a multiple of 8
    int64_t k, kb;
    int64_t chunks;        // chunks per block
    int s, b;
    int* flags;            // [0]: non-finite input seen; [1]: slice count (count-only mode)
};

constexpr int NO_ELEM = -(1 << 30);
static_assert(NO_ELEM == NO_CANDIDATE, "the two slicers share the reduction");

// Type2 codes of the two values q0 * 2^-b and q1 * 2^-b (|q| <= 2^b), packed low/high.  The hardware FP32 -> FP8
// (OCP E4M3 on gfx950) and FP32 -> FP16 conversions are exact here because every such value is a normal number of
// the format; FP32 arithmetic is not FP64 arithmetic, so the integer-only property of the slicer is about FP64.
template <int FMT>
__device__ __forceinline__ uint32_t encode_type2_pair(int q0, int q1, int b) {
    if (FMT == FMT_INT8) return ((uint32_t)q0 & 0xFFu) | (((uint32_t)q1 & 0xFFu) << 8);     // the integers themselves, |q| <= 64
    const float f0 = ldexpf((float)q0, -b), f1 = ldexpf((float)q1, -b);
    if (FMT == FMT_FP16) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const h2 h = {(_Float16)f0, (_Float16)f1};
        return __builtin_bit_cast(uint32_t, h);                       // q = 0 gives +0.0, code 0
    } else {
        const uint32_t w = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(f0, f1, 0, false) & 0xFFFFu;
        return w;
    }
}

// FP6 E2M3 code of q * 2^-(b-1), twice the slice value (|q| <= 2^b, b <= 4): with q' = q * 2^(4-b) the value is q'/8,
// and for magnitudes 0..16 the code (subnormals 0..7, normals 8..15 with exponent field 1, 16 = 2.0) is the magnitude
// itself; bit 5 is the sign.
__device__ __forceinline__ uint32_t encode_e2m3(int q, int b) {
    const int v = q << (4 - b);
    const uint32_t mag = (uint32_t)(v < 0 ? -v : v);
    return mag | (v < 0 ? 32u : 0u);
}

// FP6 E3M2 code of q * 2^-b (|q| <= 2^b, b <= 3): with q' = q * 2^(3-b) the value is q'/8; the codes (exponent field
// << 2 | fraction) of the magnitudes 0 .. 8 are 0 (zero), 2 (subnormal 2/16), 4, 6, 8, 9, 10, 11, 12; bit 5 is the sign.
__device__ __forceinline__ uint32_t encode_e3m2(int q, int b) {
    const int v = q << (3 - b);
    const uint32_t mag = (uint32_t)(v < 0 ? -v : v);
    return (uint32_t)((0xCBA986420ull >> (4 * mag)) & 0xFull) | (v < 0 ? 32u : 0u);
}

constexpr int ACTIVE = 0x7FFF;

// Element state shared by the two slicing kernels.  Dormant (not yet representable exactly with F fraction bits of
// the current unit): tv = signed 53-bit significand, pk = (E + F) | (cd << 16) with x = tv * 2^E and
// cd = ceil(log2 |x|).  Active: tv = T = x^(p) / 2^(c_p - b) * 2^F as a signed 64-bit integer (|x^(p)| <= 2^(c_p)
// bounds |T| by 2^(b+F) = 2^60), pk = ACTIVE.  An element becomes active at the first slice whose unit 2^u satisfies
// u <= E + F and stays so.
__device__ __forceinline__ void decode_element(uint64_t w, int F, int64_t& tv, int& pk, int& cmax, bool& nonfinite) {
    const int e11 = (int)((w >> 52) & 0x7FF);
    uint64_t mm = w & 0x000FFFFFFFFFFFFFull;
    nonfinite |= (e11 == 0x7FF);
    int E = -1074;
    if (e11 != 0) { mm |= 0x0010000000000000ull; E = e11 - 1075; }
    const int L = 64 - __clzll((long long)mm);                       // bit length (0 for mm == 0)
    const int cd = E + L - (((mm & (mm - 1)) == 0) ? 1 : 0);         // smallest c with |x| <= 2^c
    tv = (w >> 63) ? -(int64_t)mm : (int64_t)mm;
    pk = mm == 0 ? ACTIVE : (((E + F) & 0xFFFF) | (cd << 16));
    cmax = (mm != 0 && cd > cmax) ? cd : cmax;
}

// Eq. 5-8 for one element of an FP16 slicing and one slice whose unit is 2^unit: returns q, leaves the exact remainder
// in (T, st), and keeps track of the largest remainder of the active elements (rmax, in units of 2^(unit - F)) and of
// the largest ceil(log2 |x|) of the still dormant ones (cdorm).  rescale: left shift that brings an active remainder
// from the previous slice's unit to this one.  (Slices of at most 7 bits use slice_element.hpp instead.)
__device__ __forceinline__ int slice_element(int64_t& tv, int& pk, int unit, int rescale, int F, int64_t round_bias, uint64_t& rmax,
                                             int& cdorm) {
    // The bookkeeping of dormant elements is done with selects, the 64-bit arithmetic of active ones behind ONE
    // divergent branch: dormant elements (most of a wide-range vector during its first slices) and zeros skip it.
    const int st = pk;
    const bool was_active = st == ACTIVE;
    const int ef = (int)(short)(st & 0xFFFF);
    const bool wakes = !was_active && unit <= ef;          // representable from now on: x / 2^unit * 2^F
    const bool active = was_active || wakes;
    if (!active && unit - ef + F <= 53) {
        // With b >= 8 there are fewer than 53 fraction bits: the element reaches the unit but its low bits do not
        // fit the fixed-point form yet.  Round its integer form tv * 2^E directly, by sh = unit - E bits, and let the
        // remainder wait on as a dormant element with the same E.
        int64_t T = tv;
        const int sh = unit - ef + F;                      // F < sh <= 53
        const int64_t q64 = (T + (((int64_t)1 << (sh - 1)) - 1) + ((T >> sh) & 1)) >> sh;
        T -= q64 << sh;
        tv = T;
        const uint64_t ar = (uint64_t)(T < 0 ? -T : T);
        if (ar == 0) {
            pk = ACTIVE;                                   // nothing left: an active zero
        } else {
            const int L = 64 - __clzll((long long)ar);
            const int cd = ef - F + L - (((ar & (ar - 1)) == 0) ? 1 : 0);
            pk = (st & 0xFFFF) | (cd << 16);
            cdorm = cd > cdorm ? cd : cdorm;
        }
        return (int)q64;
    }
    const int cd = st >> 16;
    cdorm = (!active && cd > cdorm) ? cd : cdorm;          // still dormant: |x| < 2^(unit-1), q = 0, remainder = x
    pk = active ? ACTIVE : st;
    int q = 0;
    if (active) {
        // an active remainder is rescaled from the previous slice's unit, a waking element is brought to this unit
        int64_t T = tv << (was_active ? rescale : ef - unit);
        // nearest integer to T / 2^F, ties to even (two's complement form), and the exact remainder
        const int64_t q64 = (T + round_bias + ((T >> F) & 1)) >> F;
        q = (int)q64;
        T -= q64 << F;
        const uint64_t ar = (uint64_t)(T < 0 ? -T : T);
        rmax = ar > rmax ? ar : rmax;
        tv = T;
    }
    return q;
}

// Stores the Type2 codes of eight consecutive inner indices ke .. ke+7 of vector `row` into slice matrix dst_slice
// (internal layout, see layout.hpp).
template <int FMT>
__device__ __forceinline__ void store_codes(const int (&qs)[8], int64_t ke, uint8_t* dst_slice, int64_t v_rows_pad, int64_t row, int b) {
    constexpr bool FP16 = FMT == FMT_FP16;
    constexpr bool FP6 = fmt_is_fp6(FMT);
    constexpr int EPC = FP16 ? CHUNK_BYTES / 2 : CHUNK_BYTES;
    constexpr int ROWB = FP6 ? CHUNK_BYTES_FP6 : CHUNK_BYTES;
    if constexpr (FP6) {
        // eight 6-bit codes = 48 bits: octet j of the 24-byte string of k-group g, i.e. bytes
        // 6j .. 6j+5 of the string, whose first 16 bytes live in the 16-byte plane of g and the rest in the
        // 8-byte plane (see layout.hpp).  Written as one 32-bit and one 16-bit store, both naturally aligned.
        uint64_t w48 = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            w48 |= (uint64_t)(FMT == FMT_FP6_E3M2 ? encode_e3m2(qs[e], b) : encode_e2m3(qs[e], b)) << (6 * e);
        const int64_t kc = ke / EPC;
        const int o = (int)((ke % EPC) / 8), g = o >> 2, j = o & 3;
        uint8_t* const chunk = dst_slice + (size_t)kc * v_rows_pad * ROWB;
        uint8_t* const p16 = chunk + ((size_t)g * v_rows_pad + row) * 16;
        uint8_t* const p8 = chunk + (size_t)v_rows_pad * 32 + ((size_t)g * v_rows_pad + row) * 8;
        uint8_t* d32 = j == 0 ? p16 : j == 1 ? p16 + 8 : j == 2 ? p16 + 12 : p8 + 4;
        uint8_t* d16 = j == 0 ? p16 + 4 : j == 1 ? p16 + 6 : j == 2 ? p8 : p8 + 2;
        const bool low32 = (j & 1) == 0;                   // bytes 6j.. start 4-byte aligned for even j
        *reinterpret_cast<uint32_t*>(d32) = low32 ? (uint32_t)w48 : (uint32_t)(w48 >> 16);
        *reinterpret_cast<uint16_t*>(d16) = low32 ? (uint16_t)(w48 >> 32) : (uint16_t)w48;
    } else {
        uint32_t c2[4];                                            // two codes each
#pragma unroll
        for (int e = 0; e < 4; ++e) c2[e] = encode_type2_pair<FMT>(qs[2 * e], qs[2 * e + 1], b);
        const int64_t kc = ke / EPC;
        uint8_t* dst = dst_slice + ((size_t)kc * v_rows_pad + row) * CHUNK_BYTES + (ke % EPC) * (FP16 ? 2 : 1);
        if (FP16) {
            uint4 w;
            w.x = c2[0];
            w.y = c2[1];
            w.z = c2[2];
            w.w = c2[3];
            *reinterpret_cast<uint4*>(dst) = w;
        } else {
            uint2 w;
            w.x = c2[0] | (c2[1] << 16);
            w.y = c2[2] | (c2[3] << 16);
            *reinterpret_cast<uint2*>(dst) = w;
        }
    }
}

// The same for FP8 codes of the eight values qs[e] / scale (integers times a power of two, scale a power of two): the
// scaled FP32 -> FP8 pair conversion of gfx950 divides by the scale, so the slice integer is converted from where it
// sits in the slicer's upper word, without a shift or a separate scaling.  Exact for the same reason as above.
__device__ __forceinline__ void store_fp8_codes_scaled(const int (&qs)[8], float scale, int64_t ke, uint8_t* dst_slice, int64_t v_rows_pad,
                                                       int64_t row) {
    typedef short short2v __attribute__((ext_vector_type(2)));
    uint32_t w[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        short2v r = {0, 0};
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, (float)qs[4 * h], (float)qs[4 * h + 1], scale, false);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, (float)qs[4 * h + 2], (float)qs[4 * h + 3], scale, true);
        w[h] = __builtin_bit_cast(uint32_t, r);
    }
    const int64_t kc = ke / CHUNK_BYTES;
    uint8_t* dst = dst_slice + ((size_t)kc * v_rows_pad + row) * CHUNK_BYTES + (ke % CHUNK_BYTES);
    uint2 v;
    v.x = w[0];
    v.y = w[1];
    *reinterpret_cast<uint2*>(dst) = v;
}

// Where the eight 6-bit codes of one octet of a vector go inside a slice matrix: a 32-bit and a 16-bit store (see
// store_codes).  The same for every slice, so a thread works it out once per octet.
struct Fp6Slot {
    size_t at32, at16;     // byte offsets from the slice matrix
    bool low32;            // the 32-bit store takes bits 0..31 of the 48 (else bits 16..47)
};
__device__ __forceinline__ Fp6Slot fp6_slot(int64_t ke, int64_t v_rows_pad, int64_t row) {
    const int64_t kc = ke / CHUNK_BYTES;
    const int o = (int)((ke % CHUNK_BYTES) / 8), g = o >> 2, j = o & 3;
    const size_t chunk = (size_t)kc * v_rows_pad * CHUNK_BYTES_FP6;
    const size_t p16 = chunk + ((size_t)g * v_rows_pad + row) * 16;
    const size_t p8 = chunk + (size_t)v_rows_pad * 32 + ((size_t)g * v_rows_pad + row) * 8;
    Fp6Slot s;
    s.at32 = j == 0 ? p16 : j == 1 ? p16 + 8 : j == 2 ? p16 + 12 : p8 + 4;
    s.at16 = j == 0 ? p16 + 4 : j == 1 ? p16 + 6 : j == 2 ? p8 : p8 + 2;
    s.low32 = (j & 1) == 0;
    return s;
}
// FP6 codes of the eight slice integers given as q * 2^pos (the slicer's upper word), stored at a precomputed slot.
// The code of the magnitude |q| 2^(K-b) (K = 4 for E2M3, 3 for E3M2) is the magnitude itself for E2M3 and a table
// entry for E3M2 (see encode_e2m3 / encode_e3m2); bit 5 is the sign.
template <int FMT>
__device__ __forceinline__ void store_fp6_codes_at_pos(const int (&qs)[8], int pos, int b, const Fp6Slot& slot, uint8_t* dst_slice) {
    constexpr int K = FMT == FMT_FP6_E3M2 ? 3 : 4;
    const int down = pos - (K - b);
    uint32_t c[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int x = qs[e];
        const uint32_t mag = (uint32_t)(x < 0 ? -x : x) >> down;
        const uint32_t sign = ((uint32_t)x >> 26) & 32u;
        c[e] = (FMT == FMT_FP6_E3M2 ? (uint32_t)((0xCBA986420ull >> (4 * mag)) & 0xFull) : mag) | sign;
    }
    const uint32_t lo32 = c[0] | (c[1] << 6) | (c[2] << 12) | (c[3] << 18) | (c[4] << 24) | (c[5] << 30);
    const uint32_t hi16 = (c[5] >> 2) | (c[6] << 4) | (c[7] << 10);
    *reinterpret_cast<uint32_t*>(dst_slice + slot.at32) = slot.low32 ? lo32 : (lo32 >> 16) | (hi16 << 16);
    *reinterpret_cast<uint16_t*>(dst_slice + slot.at16) = (uint16_t)(slot.low32 ? hi16 : lo32);
}

// smallest c with v * 2^(unit - F) <= 2^c, for v != 0
__device__ __forceinline__ int ceil_log2_scaled(uint64_t v, int unit, int F) {
    const int L = 64 - __clzll((long long)v);
    return unit - F + L - (((v & (v - 1)) == 0) ? 1 : 0);
}

// Maximum over the 64 lanes of a wave, returned to all of them: data-parallel-primitive steps inside rows of 16 lanes
// (swap inside pairs, pairs inside quads, mirror the half rows, mirror the rows), then the last lane of a row is
// passed on to the next row(s), and lane 63 holds the maximum.
__device__ __forceinline__ int wave_max(int v) {
    auto step = [](int x, int y) { return y > x ? y : x; };
    v = step(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));      // quad_perm [1,0,3,2]
    v = step(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));      // quad_perm [2,3,0,1]
    v = step(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));     // row_half_mirror
    v = step(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false));     // row_mirror
    v = step(v, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xA, 0xF, false));     // row_bcast15 into rows 1 and 3
    v = step(v, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xC, 0xF, false));     // row_bcast31 into rows 2 and 3
    return __builtin_amdgcn_readlane(v, 63);
}

// (At least four waves per SIMD, i.e. at most 128 registers: two 512-thread workgroups per CU, so that one computes while
// the other waits at its barrier.)
template <int U, int TPR, int FMT>
__global__ void __launch_bounds__((TPR < 256 ? 256 : TPR)) __attribute__((amdgpu_waves_per_eu(4))) split_kernel(SplitArgs a) {
    constexpr bool FP16 = FMT == FMT_FP16;
    constexpr bool FP6 = fmt_is_fp6(FMT);
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int RPB = BLOCK / TPR;                  // vectors per workgroup
    constexpr int EPC = FP16 ? CHUNK_BYTES / 2 : CHUNK_BYTES;   // elements per chunk
    constexpr int ROWB = FP6 ? CHUNK_BYTES_FP6 : CHUNK_BYTES;   // bytes per vector and chunk
    constexpr int WAVES_PER_ROW = TPR / 64;
    __shared__ int red[2][BLOCK / 64];

    const int tr = threadIdx.x % TPR;
    // Workgroups are handed to the eight XCDs (each with an L2 of its own) round-robin by their index.  Neighbouring
    // vectors share the cache lines of the slice layout (a line holds the 16-byte pieces of eight vectors in the
    // FP6 planes, the 64-byte chunks of two vectors otherwise), so consecutive vectors go to workgroups of the SAME
    // XCD, where the partial lines meet in one L2 before they are written back.  Each operand's share of the grid is a multiple of 8.
    const bool second = blockIdx.x >= a.wg_first;                    // which operand this workgroup works on
    const double* const vX = second ? a.v[1].X : a.v[0].X;
    const int64_t v_ldv = second ? a.v[1].ldv : a.v[0].ldv;
    const int64_t v_rows = second ? a.v[1].rows : a.v[0].rows, v_rows_pad = second ? a.v[1].rows_pad : a.v[0].rows_pad;
    const int v_vec_ok = second ? a.v[1].vec_ok : a.v[0].vec_ok;
    uint8_t* const v_slices = second ? a.v[1].slices : a.v[0].slices;
    int32_t* const v_exps = second ? a.v[1].exps : a.v[0].exps;
    const unsigned li = blockIdx.x - (second ? a.wg_first : 0u);     // index and count inside the operand's part of the
    const unsigned gl = second ? gridDim.x - a.wg_first : a.wg_first;   // grid; both multiples of 8, so li % 8 is the XCD
    const int64_t wg = (int64_t)(li & 7) * (gl >> 3) + (li >> 3);
    const int64_t row = wg * RPB + threadIdx.x / TPR;
    const int64_t t = blockIdx.y;
    const int64_t k0 = t * a.kb;
    int64_t klen = a.k - k0;
    if (klen > a.kb) klen = a.kb;
    if (row >= v_rows) klen = 0;                      // padding vectors are all zero
    const int64_t padded = a.chunks * EPC;
    // Fixed-point scale of the working representation: an active element holds T = x^(p) / 2^(c_p - b) * 2^F as a
    // signed 64-bit integer.  |x^(p)| <= 2^(c_p) bounds |T| by 2^(b+F) = 2^60.
    const int F = 60 - a.b;

    bool nonfinite = false;
    int cmax = NO_ELEM;
    const double* src = vX + row * v_ldv + k0;
    // the eight FP64 bit patterns of octet u of this thread (zeros beyond the block)
    auto load_octet = [&](int u, uint64_t (&bits)[8]) {
        const int64_t ke = 8 * ((int64_t)tr + (int64_t)TPR * u);
        if (v_vec_ok && ke + 8 <= klen) {
            const ulonglong2* v = reinterpret_cast<const ulonglong2*>(src + ke);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                ulonglong2 w = v[h];
                bits[2 * h] = w.x;
                bits[2 * h + 1] = w.y;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) bits[e] = (ke + e < klen) ? __double_as_longlong(src[ke + e]) : 0ull;
        }
    };
    // Eq. 4: c = max over the vector of ceil(log2 |x_i|); each thread contributes the maximum over its elements
    // (from the decoded inputs for the first slice, from the remainders afterwards)
    auto vector_max = [&](int val, int p) -> int {
        static_assert(TPR >= 64, "a wave never holds parts of two vectors");
        val = wave_max(val);
        if (WAVES_PER_ROW > 1) {
            const int wave = threadIdx.x >> 6;
            if ((threadIdx.x & 63) == 0) red[p & 1][wave] = val;
            __syncthreads();
            const int w0 = (wave / WAVES_PER_ROW) * WAVES_PER_ROW;
#pragma unroll
            for (int w = 0; w < WAVES_PER_ROW; ++w) {
                const int o = red[p & 1][w0 + w];
                val = o > val ? o : val;
            }
        }
        return val;
    };

    if constexpr (!FP16) {
        // ---- slices of at most 7 bits: the element step on 32-bit words (slice_element.hpp)
        const int pos = F - 32, bias = (1 << (pos - 1)) - 1;
        const uint32_t keep = ~((1u << pos) - 1u);
        const float code_scale = ldexpf(1.0f, pos + a.b);              // q * 2^pos / code_scale = q * 2^-b, the slice value
        Fp6Slot slots[FP6 ? U : 1];                                    // FP6 only: where each octet's codes go inside a slice matrix
        if constexpr (FP6) {
#pragma unroll
            for (int u = 0; u < U; ++u) slots[u] = fp6_slot(8 * ((int64_t)tr + (int64_t)TPR * u), v_rows_pad, row);
        }
        uint64_t T[8 * U];                                             // element state, see slice_element.hpp
        int pk[8 * U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint64_t bits[8];
            load_octet(u, bits);
#pragma unroll
            for (int e = 0; e < 8; ++e) decode_narrow(bits[e], F, T[8 * u + e], pk[8 * u + e], cmax, nonfinite);
        }
        if (nonfinite) atomicOr(a.flags, 1);
        int unit_prev = 0, unit = 0, c = 0, step = 0;
        uint8_t* dst_slice = nullptr;
        int kmax, kmin;
        uint32_t cd_wait;
        // head of slice p: Eq. 4, the unit 2^(c-b) and the distance from the previous unit
        auto begin_slice = [&](int p) {
            cmax = vector_max(cmax, p);
            // count-only mode (slicing until the remainder is zero, paragraph before Eq. 4): something is left before
            // the (p+1)-th slice, so this vector needs at least p + 1 of them
            if (v_slices == nullptr && cmax != NO_ELEM && tr == 0) atomicMax(a.flags + 1, p + 1);
            c = (cmax == NO_ELEM) ? 0 : cmax;
            unit = c - a.b;
            step = unit_prev - unit;
            unit_prev = unit;
            dst_slice = v_slices + (size_t)((t * a.s + p) * a.chunks) * (size_t)v_rows_pad * ROWB;
            kmax = KEY_NONE_MAX;
            kmin = KEY_NONE_MIN;
            cd_wait = 0;
        };
        auto store_octet = [&](int u, int (&qs)[8]) {                   // qs: q * 2^pos
            const int64_t ke = 8 * ((int64_t)tr + (int64_t)TPR * u);
            if constexpr (FMT == FMT_FP8) {
                if (ke < padded && v_slices != nullptr) store_fp8_codes_scaled(qs, code_scale, ke, dst_slice, v_rows_pad, row);
            } else if constexpr (FP6) {
                if (ke < padded && v_slices != nullptr) store_fp6_codes_at_pos<FMT>(qs, pos, a.b, slots[u], dst_slice);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qs[e] >>= pos;
                if (ke < padded && v_slices != nullptr) store_codes<FMT>(qs, ke, dst_slice, v_rows_pad, row, a.b);
            }
        };
        // tail of slice p: the exponent goes out, the thread forms its candidate for the next one
        auto end_slice = [&](int p, bool settled) {
            if (tr == 0 && v_slices != nullptr) v_exps[(t * a.s + p) * v_rows_pad + row] = c;
            bool needs_exact;
            cmax = narrow_candidate(kmax, kmin, unit, F, needs_exact);
            if (needs_exact) {                                         // the upper words cannot tell: all 64 bits of the remainders
                uint64_t mx = 0;
#pragma unroll
                for (int i = 0; i < 8 * U; ++i) {
                    const uint64_t ar = (settled || pk[i] == 0) ? narrow_abs(T[i]) : 0ull;
                    mx = ar > mx ? ar : mx;
                }
                cmax = narrow_candidate_exact(mx, unit, F);
            }
            const int cw = (int)cd_wait - CD_BIAS;
            cmax = (cd_wait != 0 && cw > cmax) ? cw : cmax;
        };
        // first the slices during which some element of this wave still waits ...
        int p = 0;
        for (bool settled = false; p < a.s && !settled; ++p) {
            begin_slice(p);
            const int step16 = step * 65536;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int qs[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) qs[e] = slice_narrow(T[8 * u + e], pk[8 * u + e], step16, pos, bias, keep, kmax, kmin, cd_wait);
                store_octet(u, qs);
            }
            settled = __ballot(cd_wait != 0) == 0ull;
            end_slice(p, false);
        }
        // ... then the rest: every element is in fixed-point form, one shift for all, no control words
        for (; p < a.s; ++p) {
            begin_slice(p);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int qs[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) qs[e] = slice_narrow_active(T[8 * u + e], step, pos, bias, keep, kmax, kmin);
                store_octet(u, qs);
            }
            end_slice(p, true);
        }
        return;
    }

    // ---- FP16 slices (more than 7 bits wide): element state as described at decode_element
    int64_t tv[8 * U];
    int pk[8 * U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint64_t bits[8];
        load_octet(u, bits);
#pragma unroll
        for (int e = 0; e < 8; ++e) decode_element(bits[e], F, tv[8 * u + e], pk[8 * u + e], cmax, nonfinite);
    }
    if (nonfinite) atomicOr(a.flags, 1);

    int c_prev = 0;
    for (int p = 0; p < a.s; ++p) {
        cmax = vector_max(cmax, p);
        if (v_slices == nullptr) {
            if (cmax != NO_ELEM && tr == 0) atomicMax(a.flags + 1, p + 1);      // count-only mode
        }
        const int c = (cmax == NO_ELEM) ? 0 : cmax;
        const int unit = c - a.b;                                      // the slice's unit is 2^(c-b)
        // remainders of active elements were left in units of the previous slice: rescale them to this one (a
        // left shift, exact and inside 2^60 because every remainder is at most 2^c; 0 << anything stays 0)
        int rescale = p == 0 ? 0 : c_prev - c;
        rescale = rescale < 0 ? 0 : (rescale > 63 ? 63 : rescale);
        c_prev = c;

        // ---- Eq. 5-8 element by element, eight codes per store
        uint8_t* const dst_slice = v_slices + (size_t)((t * a.s + p) * a.chunks) * (size_t)v_rows_pad * ROWB;
        uint64_t rmax = 0;                                             // largest |remainder| of this thread's active elements
        int cdorm = NO_ELEM;                                           // largest cd of its still dormant elements
        const int64_t round_bias = ((int64_t)1 << (F - 1)) - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int qs[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) qs[e] = slice_element(tv[8 * u + e], pk[8 * u + e], unit, rescale, F, round_bias, rmax, cdorm);
            const int64_t ke = 8 * ((int64_t)tr + (int64_t)TPR * u);
            if (ke < padded && v_slices != nullptr) store_codes<FMT>(qs, ke, dst_slice, v_rows_pad, row, a.b);
        }
        if (tr == 0 && v_slices != nullptr) v_exps[(t * a.s + p) * v_rows_pad + row] = c;
        // this thread's candidate for the next exponent: remainders are rmax * 2^(unit - F)
        cmax = cdorm;
        if (rmax != 0) {
            const int ca = ceil_log2_scaled(rmax, unit, F);
            cmax = ca > cmax ? ca : cmax;
        }
    }
}

// The same slicing for blocks too long for the registers of one workgroup: one workgroup of 1024 threads per vector
// and block streams through the vector once per slice, with the element state (decode_element) kept in work memory
// between the slices: tv_state / pk_state hold one int64 / int32 per element of the (real) vectors.
template <int FMT>
__global__ void __launch_bounds__(1024) split_stream_kernel(SplitArgs a, int64_t* tv_state, int* pk_state) {
    constexpr bool FP16 = FMT == FMT_FP16;
    constexpr int EPC = FP16 ? CHUNK_BYTES / 2 : CHUNK_BYTES;
    constexpr int ROWB = fmt_is_fp6(FMT) ? CHUNK_BYTES_FP6 : CHUNK_BYTES;
    __shared__ int red[2][16];
    const int tid = threadIdx.x, wave = tid >> 6;
    const bool second = blockIdx.x >= a.wg_first;
    const SplitVectors& v = second ? a.v[1] : a.v[0];
    const int64_t row = blockIdx.x - (second ? a.wg_first : 0u);
    const int64_t t = blockIdx.y, T = gridDim.y;
    const int64_t k0 = t * a.kb;
    int64_t klen = a.k - k0;
    if (klen > a.kb) klen = a.kb;
    const int64_t padded = a.chunks * EPC, n_oct = padded / 8;
    const int F = 60 - a.b;
    if (row >= v.rows) {
        // a padding vector: zero codes and c = 0 in every slice
        if (v.slices == nullptr) return;
        const int zero8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int p = 0; p < a.s; ++p) {
            uint8_t* const dst_slice = v.slices + (size_t)((t * a.s + p) * a.chunks) * (size_t)v.rows_pad * ROWB;
            for (int64_t o = tid; o < n_oct; o += 1024) store_codes<FMT>(zero8, 8 * o, dst_slice, v.rows_pad, row, a.b);
            if (tid == 0) v.exps[(t * a.s + p) * v.rows_pad + row] = 0;
        }
        return;
    }
    // this vector's state: real vectors of the first operand, then those of the second, each with T blocks
    const int64_t vec = (second ? a.v[0].rows : 0) + row;
    int64_t* const tv = tv_state + (size_t)(vec * T + t) * padded;
    int* const pk = pk_state + (size_t)(vec * T + t) * padded;

    // block-wide maximum of an int, double-buffered so that one barrier per reduction suffices
    int round = 0;
    auto block_max = [&](int val) -> int {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_xor(val, off, 64);
            val = o > val ? o : val;
        }
        if ((tid & 63) == 0) red[round & 1][wave] = val;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int o = red[round & 1][w];
            val = o > val ? o : val;
        }
        ++round;
        return val;
    };

    bool nonfinite = false;
    int cmax = NO_ELEM;
    const double* src = v.X + row * v.ldv + k0;
    if constexpr (!FP16) {
        // ---- slices of at most 7 bits: the 32-bit element step of slice_element.hpp, state = (T, control word)
        uint64_t* const Ts = reinterpret_cast<uint64_t*>(tv);
        const int pos = F - 32, bias = (1 << (pos - 1)) - 1;
        const uint32_t keep = ~((1u << pos) - 1u);
        for (int64_t o = tid; o < n_oct; o += 1024) {
            const int64_t ke = 8 * o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t w = (ke + e < klen) ? (uint64_t)__double_as_longlong(src[ke + e]) : 0ull;
                uint64_t T0;
                int st;
                decode_narrow(w, F, T0, st, cmax, nonfinite);
                Ts[ke + e] = T0;
                pk[ke + e] = st;
            }
        }
        if (nonfinite) atomicOr(a.flags, 1);
        cmax = block_max(cmax);
        int unit_prev = 0;
        for (int p = 0; p < a.s; ++p) {
            if (v.slices == nullptr && cmax != NO_ELEM && tid == 0) atomicMax(a.flags + 1, p + 1);     // count-only mode
            const int c = (cmax == NO_ELEM) ? 0 : cmax;
            const int unit = c - a.b;
            const int step16 = (unit_prev - unit) * 65536;
            unit_prev = unit;
            uint8_t* const dst_slice = v.slices + (size_t)((t * a.s + p) * a.chunks) * (size_t)v.rows_pad * ROWB;
            int kmax = KEY_NONE_MAX, kmin = KEY_NONE_MIN;
            uint32_t cd_wait = 0;
            for (int64_t o = tid; o < n_oct; o += 1024) {
                const int64_t ke = 8 * o;
                int qs[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    uint64_t T0 = Ts[ke + e];
                    int st = pk[ke + e];
                    qs[e] = slice_narrow(T0, st, step16, pos, bias, keep, kmax, kmin, cd_wait) >> pos;
                    Ts[ke + e] = T0;
                    pk[ke + e] = st;
                }
                if (v.slices != nullptr) store_codes<FMT>(qs, ke, dst_slice, v.rows_pad, row, a.b);
            }
            if (tid == 0 && v.slices != nullptr) v.exps[(t * a.s + p) * v.rows_pad + row] = c;
            bool needs_exact;
            cmax = narrow_candidate(kmax, kmin, unit, F, needs_exact);
            if (needs_exact) {                                         // the upper words cannot tell: once more through the state
                uint64_t mx = 0;
                for (int64_t o = tid; o < n_oct; o += 1024)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint64_t ar = pk[8 * o + e] == 0 ? narrow_abs(Ts[8 * o + e]) : 0ull;
                        mx = ar > mx ? ar : mx;
                    }
                cmax = narrow_candidate_exact(mx, unit, F);
            }
            const int cw = (int)cd_wait - CD_BIAS;
            cmax = (cd_wait != 0 && cw > cmax) ? cw : cmax;
            cmax = block_max(cmax);
        }
        return;
    }
    // ---- FP16 slices: the 64-bit element step (decode_element / slice_element)
    for (int64_t o = tid; o < n_oct; o += 1024) {
        const int64_t ke = 8 * o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint64_t w = (ke + e < klen) ? (uint64_t)__double_as_longlong(src[ke + e]) : 0ull;
            int64_t T0;
            int st;
            decode_element(w, F, T0, st, cmax, nonfinite);
            tv[ke + e] = T0;
            pk[ke + e] = st;
        }
    }
    if (nonfinite) atomicOr(a.flags, 1);
    cmax = block_max(cmax);

    int c_prev = 0;
    for (int p = 0; p < a.s; ++p) {
        if (v.slices == nullptr && cmax != NO_ELEM && tid == 0) atomicMax(a.flags + 1, p + 1);     // count-only mode
        const int c = (cmax == NO_ELEM) ? 0 : cmax;
        const int unit = c - a.b;
        int rescale = p == 0 ? 0 : c_prev - c;
        rescale = rescale < 0 ? 0 : (rescale > 63 ? 63 : rescale);
        c_prev = c;
        uint8_t* const dst_slice = v.slices + (size_t)((t * a.s + p) * a.chunks) * (size_t)v.rows_pad * ROWB;
        uint64_t rmax = 0;
        int cdorm = NO_ELEM;
        const int64_t round_bias = ((int64_t)1 << (F - 1)) - 1;
        for (int64_t o = tid; o < n_oct; o += 1024) {
            const int64_t ke = 8 * o;
            int qs[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int64_t T0 = tv[ke + e];
                int st = pk[ke + e];
                qs[e] = slice_element(T0, st, unit, rescale, F, round_bias, rmax, cdorm);
                tv[ke + e] = T0;
                pk[ke + e] = st;
            }
            if (v.slices != nullptr) store_codes<FMT>(qs, ke, dst_slice, v.rows_pad, row, a.b);
        }
        if (tid == 0 && v.slices != nullptr) v.exps[(t * a.s + p) * v.rows_pad + row] = c;
        cmax = cdorm;
        if (rmax != 0) {
            const int ca = ceil_log2_scaled(rmax, unit, F);
            cmax = ca > cmax ? ca : cmax;
        }
        cmax = block_max(cmax);
    }
}

template <int FMT>
__global__ void __launch_bounds__(256) export_slices_kernel(const uint8_t* __restrict__ slices, int64_t rows, int64_t rows_pad,
                                                            int64_t k, int64_t kb, int64_t chunks, int s, void* out) {
    // plain layout: block t starts at s*rows*(t*kb) entries; inside, [p][row][kb_t]
    constexpr bool FP16 = FMT == FMT_FP16;
    constexpr bool FP6 = fmt_is_fp6(FMT);
    constexpr int EPC = FP16 ? CHUNK_BYTES / 2 : CHUNK_BYTES;
    constexpr int ROWB = FP6 ? CHUNK_BYTES_FP6 : CHUNK_BYTES;
    const int64_t t = blockIdx.z, p = blockIdx.y;
    int64_t klen = k - t * kb;
    if (klen > kb) klen = kb;
    const int64_t total = rows * klen;
    const uint8_t* src = slices + (size_t)((t * s + p) * chunks) * (size_t)rows_pad * ROWB;
    const size_t out_base = (size_t)s * rows * (t * kb) + (size_t)p * rows * klen;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / klen, kk = idx % klen;
        if constexpr (FP6) {
            // code i of k-group g sits at bits 6i .. 6i+5 of a 24-byte string: bytes 0..15 in the 16-byte plane of g,
            // bytes 16..23 in its 8-byte plane
            const uint8_t* chunk = src + (size_t)(kk / EPC) * rows_pad * ROWB;
            const int e = (int)(kk % EPC), g = e >> 5, bit = (e & 31) * 6;
            const uint8_t* p16 = chunk + ((size_t)g * rows_pad + r) * 16;
            const uint8_t* p8 = chunk + (size_t)rows_pad * 32 + ((size_t)g * rows_pad + r) * 8;
            const int b0 = bit >> 3, b1 = (bit + 5) >> 3;
            const uint32_t lo = b0 < 16 ? p16[b0] : p8[b0 - 16], hi = b1 < 16 ? p16[b1] : p8[b1 - 16];
            reinterpret_cast<uint8_t*>(out)[out_base + idx] = (uint8_t)((((hi << 8) | lo) >> (bit & 7)) & 63u);
        } else {
            const size_t off = ((size_t)(kk / EPC) * rows_pad + r) * CHUNK_BYTES + (kk % EPC) * (FP16 ? 2 : 1);
            if (FP16) reinterpret_cast<uint16_t*>(out)[out_base + idx] = *reinterpret_cast<const uint16_t*>(src + off);
            else reinterpret_cast<uint8_t*>(out)[out_base + idx] = src[off];
        }
    }
}

// One workgroup per 256 vectors and block, one half-wave per group of 32 vectors: for every slice p, is c_p - c_(p+1)
// the same for all real vectors of the group?  The first tiles_first workgroups of a grid row belong to the first
// operand, the rest to the second.
struct DeltaOperand {
    const int32_t* exps;
    int32_t* deltas;
    int64_t rows, rows_pad;
};
__global__ void __launch_bounds__(256) delta_kernel(DeltaOperand o0, DeltaOperand o1, unsigned tiles_first, int s) {
    const bool second = blockIdx.x >= tiles_first;
    const int32_t* const exps = second ? o1.exps : o0.exps;
    int32_t* const deltas = second ? o1.deltas : o0.deltas;
    const int64_t rows = second ? o1.rows : o0.rows, rows_pad = second ? o1.rows_pad : o0.rows_pad;
    const int64_t tile = blockIdx.x - (second ? tiles_first : 0u), groups = rows_pad / LINK_ROWS, t = blockIdx.y;
    const int64_t row = tile * TILE + threadIdx.x;
    const int64_t group = row / LINK_ROWS;
    const int lane = threadIdx.x & 63, half = lane & 32;
    const int32_t* e = exps + (size_t)t * s * rows_pad;
    int32_t* out = deltas + (size_t)t * s * groups + group;          // slice p of this group at out[p * groups]
    for (int p = 0; p + 1 < s; ++p) {
        const int d = e[(size_t)p * rows_pad + row] - e[(size_t)(p + 1) * rows_pad + row];
        // the first vector of a group is a real one, or the whole group is padding (then every d is 0)
        const int ref = __shfl(d, half, 64);
        const unsigned long long ok = __ballot(row >= rows || d == ref);
        const bool same = (uint32_t)(ok >> half) == 0xFFFFFFFFu;
        if ((lane & 31) == 0) out[(size_t)p * groups] = same ? ref : DELTA_IRREGULAR;
    }
    if ((lane & 31) == 0) out[(size_t)(s - 1) * groups] = DELTA_IRREGULAR;
}

template <int U, int TPR>
hipError_t launch_split_cfg(const SplitArgs& a_in, int fmt, int64_t T, hipStream_t st) {
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int RPB = BLOCK / TPR;
    SplitArgs a = a_in;
    a.wg_first = (unsigned)(a.v[0].rows_pad / RPB);                     // rows_pad is a multiple of 256, RPB <= 4
    dim3 grid(a.wg_first + (unsigned)(a.v[1].rows_pad / RPB), (unsigned)T);
    if (fmt == FMT_FP16) hipLaunchKernelGGL((split_kernel<U, TPR, FMT_FP16>), grid, dim3(BLOCK), 0, st, a);
    else if (fmt == FMT_FP6) hipLaunchKernelGGL((split_kernel<U, TPR, FMT_FP6>), grid, dim3(BLOCK), 0, st, a);
    else if (fmt == FMT_FP6_E3M2) hipLaunchKernelGGL((split_kernel<U, TPR, FMT_FP6_E3M2>), grid, dim3(BLOCK), 0, st, a);
    else if (fmt == FMT_INT8) hipLaunchKernelGGL((split_kernel<U, TPR, FMT_INT8>), grid, dim3(BLOCK), 0, st, a);
    else hipLaunchKernelGGL((split_kernel<U, TPR, FMT_FP8>), grid, dim3(BLOCK), 0, st, a);
    return hipGetLastError();
}

// blocks too long for the register-resident kernel: one workgroup per vector (real and padding) and block
hipError_t launch_split_stream(const SplitArgs& a_in, int fmt, int64_t T, void* state, hipStream_t st) {
    if (state == nullptr) return hipErrorInvalidValue;
    SplitArgs a = a_in;
    a.wg_first = (unsigned)a.v[0].rows_pad;
    const int64_t elems = (a.v[0].rows + a.v[1].rows) * T * a.chunks * (fmt == FMT_FP16 ? CHUNK_BYTES / 2 : CHUNK_BYTES);
    int64_t* tv = static_cast<int64_t*>(state);
    int* pk = reinterpret_cast<int*>(tv + elems);
    dim3 grid(a.wg_first + (unsigned)a.v[1].rows_pad, (unsigned)T);
    if (fmt == FMT_FP16) hipLaunchKernelGGL((split_stream_kernel<FMT_FP16>), grid, dim3(1024), 0, st, a, tv, pk);
    else if (fmt == FMT_FP6) hipLaunchKernelGGL((split_stream_kernel<FMT_FP6>), grid, dim3(1024), 0, st, a, tv, pk);
    else if (fmt == FMT_FP6_E3M2) hipLaunchKernelGGL((split_stream_kernel<FMT_FP6_E3M2>), grid, dim3(1024), 0, st, a, tv, pk);
    else if (fmt == FMT_INT8) hipLaunchKernelGGL((split_stream_kernel<FMT_INT8>), grid, dim3(1024), 0, st, a, tv, pk);
    else hipLaunchKernelGGL((split_stream_kernel<FMT_FP8>), grid, dim3(1024), 0, st, a, tv, pk);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_transpose(const double* A, int64_t lda, int64_t m, int64_t k, double* At, hipStream_t st) {
    if (m == 0 || k == 0) return hipSuccess;
    dim3 grid((unsigned)((m + 31) / 32), (unsigned)((k + 31) / 32));
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, st, A, lda, m, k, At);
    return hipGetLastError();
}

namespace {
SplitVectors split_vectors(const double* X, int64_t ldv, const Plan& pl, const Operand* op) {
    SplitVectors v;
    memset(&v, 0, sizeof(v));
    if (op == nullptr || op->rows == 0) return v;                                 // no vectors: no workgroups
    v.X = X; v.ldv = ldv; v.rows = op->rows; v.rows_pad = op->rows_pad; v.slices = op->slices; v.exps = op->exps;
    v.vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0) && (ldv % 2 == 0) && (pl.kb % 2 == 0 || pl.T == 1);
    return v;
}
}  // namespace

size_t split_state_bytes(const Plan& pl, int64_t rows_a, int64_t rows_b) {
    if (pl.kb <= MAX_K_BLOCK_IN_REGISTERS) return 0;
    return (size_t)(rows_a + rows_b) * pl.T * pl.chunks * pl.epc * (sizeof(int64_t) + sizeof(int));
}

hipError_t launch_split(const double* X0, int64_t ldv0, const Operand* op0, const double* X1, int64_t ldv1, const Operand* op1,
                        const Plan& pl, int* flags, void* long_state, hipStream_t st) {
    SplitArgs a;
    a.v[0] = split_vectors(X0, ldv0, pl, op0);
    a.v[1] = split_vectors(X1, ldv1, pl, op1);
    a.wg_first = 0;
    a.k = pl.k; a.kb = pl.kb; a.chunks = pl.chunks; a.s = pl.s; a.b = pl.b; a.flags = flags;
    if (a.v[0].rows_pad + a.v[1].rows_pad == 0 || pl.T == 0) return hipSuccess;
    const int64_t vectors = (a.v[0].rows_pad + a.v[1].rows_pad) * pl.T;
    const int fmt = pl.fmt;
    if (pl.kb > MAX_K_BLOCK_IN_REGISTERS) return launch_split_stream(a, fmt, pl.T, long_state, st);
    const int64_t octets = pl.chunks * pl.epc / 8;                              // per vector and block, padded
    // sixteen elements per thread (U = 2) is the measured optimum: more elements per thread cost registers and with
    // them the occupancy that hides the latency of the dependent integer chains (64 per thread: one wave per SIMD)
    if (octets <= 64) return launch_split_cfg<1, 64>(a, fmt, pl.T, st);
    // a small problem (few vectors) is bound by the length of a thread's dependent chain, not by throughput: eight
    // elements per thread there (1024 x 1024: 0.080 -> 0.065 ms for both operands; no gain from 2048 vectors on)
    if (vectors <= 2048) {
        if (octets <= 128) return launch_split_cfg<1, 128>(a, fmt, pl.T, st);
        if (octets <= 256) return launch_split_cfg<1, 256>(a, fmt, pl.T, st);
    }
    if (octets <= 128) return launch_split_cfg<2, 64>(a, fmt, pl.T, st);
    if (octets <= 256) return launch_split_cfg<2, 128>(a, fmt, pl.T, st);
    if (octets <= 512) return launch_split_cfg<2, 256>(a, fmt, pl.T, st);
    if (octets <= 1024) return launch_split_cfg<2, 512>(a, fmt, pl.T, st);
    if (octets <= 2048) return launch_split_cfg<2, 1024>(a, fmt, pl.T, st);
    // 32 elements per thread would cover blocks of up to 32768 elements, but at the 128 registers a thread of a
    // 1024-thread workgroup has, that variant lives on more than a hundred spilled registers; such blocks are streamed
    return hipErrorInvalidValue;
}

hipError_t launch_count_slices(const double* X, int64_t ldv, const Plan& pl, int64_t rows, int* flags, void* long_state, hipStream_t st) {
    Plan cp = pl;
    cp.s = MAX_SLICES + 1;                       // one more than the library can use: "not exhausted" is reported as 33
    Operand op;
    op.rows = rows;
    op.rows_pad = (rows + TILE - 1) / TILE * TILE;
    op.slices = nullptr; op.exps = nullptr; op.deltas = nullptr;
    return launch_split(X, ldv, &op, nullptr, 0, nullptr, cp, flags, long_state, st);
}

hipError_t launch_deltas(const Plan& pl, const Operand* op0, const Operand* op1, hipStream_t st) {
    DeltaOperand o[2];
    memset(o, 0, sizeof(o));
    const Operand* ops[2] = {op0, op1};
    for (int i = 0; i < 2; ++i)
        if (ops[i] != nullptr && ops[i]->rows > 0) o[i] = DeltaOperand{ops[i]->exps, ops[i]->deltas, ops[i]->rows, ops[i]->rows_pad};
    const unsigned t0 = (unsigned)(o[0].rows_pad / TILE), t1 = (unsigned)(o[1].rows_pad / TILE);
    if (t0 + t1 == 0 || pl.T == 0 || pl.s == 0) return hipSuccess;
    hipLaunchKernelGGL(delta_kernel, dim3(t0 + t1, (unsigned)pl.T), dim3(256), 0, st, o[0], o[1], t0, pl.s);
    return hipGetLastError();
}

hipError_t launch_export_slices(const Plan& pl, const Operand& op, void* out, hipStream_t st) {
    if (op.rows == 0 || pl.k == 0) return hipSuccess;
    dim3 grid(1024, (unsigned)pl.s, (unsigned)pl.T);
    if (pl.fmt == FMT_FP16)
        hipLaunchKernelGGL((export_slices_kernel<FMT_FP16>), grid, dim3(256), 0, st, op.slices, op.rows, op.rows_pad, pl.k, pl.kb, pl.chunks, pl.s, out);
    else if (fmt_is_fp6(pl.fmt))
        hipLaunchKernelGGL((export_slices_kernel<FMT_FP6>), grid, dim3(256), 0, st, op.slices, op.rows, op.rows_pad, pl.k, pl.kb, pl.chunks, pl.s, out);
    else
        hipLaunchKernelGGL((export_slices_kernel<FMT_FP8>), grid, dim3(256), 0, st, op.slices, op.rows, op.rows_pad, pl.k, pl.kb, pl.chunks, pl.s, out);
    return hipGetLastError();
}

}  // namespace ozaki
