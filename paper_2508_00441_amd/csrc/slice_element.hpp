// The per-element step of the slicer for formats whose slices are at most 7 bits wide (FP8, FP6, INT8): Eq. 5-8 of
// the paper on a 64-bit fixed-point number held as two 32-bit words, so that the rounding, the subtraction and the
// bookkeeping for the next exponent are 32-bit integer operations.
//
// With F = 60 - b fraction bits (F >= 53 here) an element of slice p is T = x^(p) / 2^(c_p - b) * 2^F, |T| <= 2^60.
// The unit of the slice sits at bit F of T, i.e. at bit pos = F - 32 of the upper word:
//     q        = nearest integer to T / 2^F, ties to even: (hi + (2^(pos-1) - 1) + carry) >> pos, where the carry out
//                of the lower word of T + (2^(F-1) - 1) + (unit bit of T) is (lo != 0) | unit bit
//     T - q 2^F  changes the upper word only
// What the next exponent needs of a remainder is ceil(log2 |T|).  It is read off the 32-bit key |2 hi + (lo != 0)|,
// which has the same ceil(log2) as |T| / 2^31 whenever |T| >= 2^32; a thread whose remainders are all smaller falls
// back to the lower words (narrow_small_abs).
//
// An element whose lowest bit lies below 2^-F of the current unit cannot be written this way yet (it is then smaller
// than an eighth of the unit: q = 0).  It waits with its significand in (hi, lo); the control word pk holds
//     upper half: E + F - u, the left shift that would bring the significand to the unit 2^u of the current slice
//                 (negative while waiting), for x = significand * 2^E
//     lower half: ceil(log2 |x|) + CD_BIAS while waiting, 0 afterwards
// and every slice adds (u_previous - u) to the upper half: for an element that is already in fixed-point form (upper
// half left at 0) that is exactly the left shift from the previous unit to this one, so one rule serves both.
//
// Compiles for the device and, for CPU-side unit tests of this very code, for the host.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define OZAKI_SLICE_HD __host__ __device__ __forceinline__
#else
#define OZAKI_SLICE_HD inline
#endif

namespace ozaki {

constexpr int CD_BIAS = 2048;             // ceil(log2 |x|) of a finite FP64 number is in [-1074, 1024]
constexpr int NO_CANDIDATE = -(1 << 30);

OZAKI_SLICE_HD int bit_length_u64(uint64_t v) {            // 0 for v == 0
#if defined(__HIP_DEVICE_COMPILE__)
    return 64 - __clzll((long long)v);
#else
    return v ? 64 - __builtin_clzll(v) : 0;
#endif
}
OZAKI_SLICE_HD int bit_length_u32(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return 32 - __clz((int)v);
#else
    return v ? 32 - __builtin_clz(v) : 0;
#endif
}

// FP64 bits -> waiting element.  cmax collects ceil(log2 |x|) over the non-zero elements.
OZAKI_SLICE_HD void decode_narrow(uint64_t w, int F, int& hi, uint32_t& lo, int& pk, int& cmax, bool& nonfinite) {
    const int e11 = (int)((w >> 52) & 0x7FF);
    uint64_t mm = w & 0x000FFFFFFFFFFFFFull;
    nonfinite |= (e11 == 0x7FF);
    int E = -1074;
    if (e11 != 0) { mm |= 0x0010000000000000ull; E = e11 - 1075; }
    const int cd = E + bit_length_u64(mm) - (((mm & (mm - 1)) == 0) ? 1 : 0);     // smallest c with |x| <= 2^c
    const int64_t tv = (w >> 63) ? -(int64_t)mm : (int64_t)mm;
    hi = (int)(tv >> 32);
    lo = (uint32_t)tv;
    pk = mm == 0 ? 0 : (E + F) * 65536 + (cd + CD_BIAS);
    cmax = (mm != 0 && cd > cmax) ? cd : cmax;
}

// One element, one slice.  step16 = (previous unit - this unit) * 65536 (minus this unit for the first slice);
// pos = F - 32, bias = 2^(pos-1) - 1, keep = ~(2^pos - 1).  Returns q * 2^pos (the slice integer where it sits in the
// upper word); kmax / kmin collect the signed keys of the remainders, cd_wait the largest lower half of the elements
// that go on waiting.
OZAKI_SLICE_HD int slice_narrow(int& hi, uint32_t& lo, int& pk, int step16, int pos, int bias, uint32_t keep, int& kmax, int& kmin,
                                uint32_t& cd_wait) {
    pk += step16;
    int q_at_pos = 0;
    if (pk >= 0) {
        const int sh = pk >> 16;                                     // 0 .. 60: nothing is shifted out (|T| <= 2^60 afterwards)
        const uint64_t T = (((uint64_t)(uint32_t)hi << 32) | lo) << (sh & 63);
        hi = (int)(uint32_t)(T >> 32);
        lo = (uint32_t)T;
        const int nz = lo != 0 ? 1 : 0;
        const int sum = hi + bias + (nz | ((hi >> pos) & 1));
        q_at_pos = (int)((uint32_t)sum & keep);
        hi -= q_at_pos;
        const int key = (int)(((uint32_t)hi << 1) | (uint32_t)nz);
        kmax = key > kmax ? key : kmax;
        kmin = key < kmin ? key : kmin;
        pk = 0;
    }
    const uint32_t cdw = (uint32_t)pk & 0xFFFFu;                     // 0 unless the element goes on waiting
    cd_wait = cdw > cd_wait ? cdw : cd_wait;
    return q_at_pos;
}

// |T| of a remainder known to be below 2^32 in magnitude (key 0 or 1)
OZAKI_SLICE_HD uint32_t narrow_small_abs(int hi, uint32_t lo) { return hi < 0 ? 0u - lo : lo; }

// The candidate for the next exponent from a thread's keys: smallest c with (largest |T|) * 2^(unit - F) <= 2^c, or
// NO_CANDIDATE for no remainder at all.  needs_low is set when the keys cannot tell (largest key 1): the caller then
// passes the largest narrow_small_abs of its elements to narrow_candidate_low.
OZAKI_SLICE_HD int narrow_candidate(int kmax, int kmin, int unit, int F, bool& needs_low) {
    const int K = kmax > -kmin ? kmax : -kmin;
    needs_low = K == 1;
    if (K < 2) return NO_CANDIDATE;
    return unit - F + 31 + bit_length_u32((uint32_t)K - 1u);          // ceil(log2 K) for K >= 2
}
OZAKI_SLICE_HD int narrow_candidate_low(uint32_t max_abs, int unit, int F) {
    if (max_abs == 0) return NO_CANDIDATE;
    return unit - F + (max_abs == 1 ? 0 : bit_length_u32(max_abs - 1u));
}

}  // namespace ozaki
