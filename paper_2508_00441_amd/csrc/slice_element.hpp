// The per-element step of the slicer for formats whose slices are at most 7 bits wide (FP8, FP6, INT8): Eq. 5-8 of
// the paper on a 64-bit fixed-point number held as two 32-bit words, so that the rounding, the subtraction and the
// bookkeeping for the next exponent are 32-bit integer operations.
//
// With F = 60 - b fraction bits (F >= 53 here) an element of slice p is T = x^(p) / 2^(c_p - b) * 2^F, |T| <= 2^60.
// The unit of the slice sits at bit F of T, i.e. at bit pos = F - 32 of the upper word:
//     q        = nearest integer to T / 2^F, ties to even: (hi + (2^(pos-1) - 1) + carry) >> pos, where the carry out
//                of the lower word of T + (2^(F-1) - 1) + (unit bit of T) is (lo != 0) | unit bit
//     T - q 2^F  changes the upper word only
// What the next exponent needs of the remainders is ceil(log2 max|T|).  The thread keeps the largest and the smallest
// upper word of its remainders: an upper word h > 0 means h 2^32 <= |T| < (h+1) 2^32, an upper word -n < 0 means
// (n-1) 2^32 < |T| <= n 2^32, so the two extremes fix ceil(log2) unless the largest positive upper word is a power
// of two (then the lower word of that element decides) or every remainder is below 2^32 in magnitude; in those
// cases the thread goes through its elements once more with the full 64 bits (narrow_abs).
//
// An element whose lowest bit lies below 2^-F of the current unit cannot be written this way yet (it is then smaller
// than an eighth of the unit: q = 0).  It waits with its significand in T; the control word pk holds
//     upper half: E + F - u, the left shift that would bring the significand to the unit 2^u of the current slice
//                 (negative while waiting), for x = significand * 2^E
//     lower half: ceil(log2 |x|) + CD_BIAS while waiting, 0 afterwards
// (a zero element is in fixed-point form from the start) and every slice adds (u_previous - u) to the upper half: for an element that is already in fixed-point form (upper
// half left at 0) that is exactly the left shift from the previous unit to this one, so one rule serves both.
// Once no element of a wave waits any more, the control words are dropped and the shift is the same for all
// (slice_narrow_active).
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
OZAKI_SLICE_HD void decode_narrow(uint64_t w, int F, uint64_t& T, int& pk, int& cmax, bool& nonfinite) {
    const int e11 = (int)((w >> 52) & 0x7FF);
    uint64_t mm = w & 0x000FFFFFFFFFFFFFull;
    nonfinite |= (e11 == 0x7FF);
    int E = -1074;
    if (e11 != 0) { mm |= 0x0010000000000000ull; E = e11 - 1075; }
    const int cd = E + bit_length_u64(mm) - (((mm & (mm - 1)) == 0) ? 1 : 0);     // smallest c with |x| <= 2^c
    T = (w >> 63) ? 0ull - mm : mm;                                  // two's complement
    pk = mm == 0 ? 2047 * 65536 : (E + F) * 65536 + (cd + CD_BIAS);      // zero: in fixed-point form whatever the first unit is
    cmax = (mm != 0 && cd > cmax) ? cd : cmax;
}

constexpr int KEY_NONE_MAX = -0x7FFFFFFF - 1, KEY_NONE_MIN = 0x7FFFFFFF;      // initial kmax / kmin: no remainder seen

// Eq. 5-8 on an element in fixed-point form whose remainder is still in units of the previous slice: `shift` brings it
// to this slice's unit.  pos = F - 32, bias = 2^(pos-1) - 1, keep = ~(2^pos - 1).  Returns q * 2^pos (the slice integer
// where it sits in the upper word); kmax / kmin collect the upper words of the remainders.
OZAKI_SLICE_HD int slice_narrow_active(uint64_t& T, int shift, int pos, int bias, uint32_t keep, int& kmax, int& kmin) {
    const uint64_t t = T << (shift & 63);                           // nothing is shifted out: |T| <= 2^60 afterwards
    int hi = (int)(uint32_t)(t >> 32);
    const uint32_t lo = (uint32_t)t;
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t nz;                                                    // lo != 0 as 0 / 1: one 32-bit minimum (written out because
    asm("v_min_u32 %0, 1, %1" : "=v"(nz) : "v"(lo));                // the compiler turns the C form into a 64-bit compare and a select)
#else
    const uint32_t nz = lo != 0 ? 1u : 0u;
#endif
    const uint32_t carry = nz | (((uint32_t)hi >> pos) & 1u);       // (lo != 0) | unit bit
    const int sum = hi + bias + (int)carry;
    const int q_at_pos = (int)((uint32_t)sum & keep);
    hi -= q_at_pos;
    kmax = hi > kmax ? hi : kmax;
    kmin = hi < kmin ? hi : kmin;
    T = ((uint64_t)(uint32_t)hi << 32) | lo;
    return q_at_pos;
}

// One element that may still be waiting, one slice.  step16 = (previous unit - this unit) * 65536 (minus this unit for
// the first slice).  cd_wait collects the largest lower half of the elements that go on waiting.
OZAKI_SLICE_HD int slice_narrow(uint64_t& T, int& pk, int step16, int pos, int bias, uint32_t keep, int& kmax, int& kmin,
                                uint32_t& cd_wait) {
    pk += step16;
    int q_at_pos = 0;
    if (pk >= 0) {
        q_at_pos = slice_narrow_active(T, pk >> 16, pos, bias, keep, kmax, kmin);
        pk = 0;
    }
    const uint32_t cdw = (uint32_t)pk & 0xFFFFu;                     // 0 unless the element goes on waiting
    cd_wait = cdw > cd_wait ? cdw : cd_wait;
    return q_at_pos;
}

// |T| of a remainder
OZAKI_SLICE_HD uint64_t narrow_abs(uint64_t T) { return (int64_t)T < 0 ? 0ull - T : T; }

// The candidate for the next exponent from a thread's extreme upper words: smallest c with (largest |T|) *
// 2^(unit - F) <= 2^c, NO_CANDIDATE if the thread has no remainder.  needs_exact is set when the upper words cannot
// tell: the caller then passes the largest narrow_abs of its elements in fixed-point form to narrow_candidate_exact.
OZAKI_SLICE_HD int narrow_candidate(int kmax, int kmin, int unit, int F, bool& needs_exact) {
    needs_exact = false;
    if (kmax == KEY_NONE_MAX) return NO_CANDIDATE;
    const uint32_t P = kmax > 0 ? (uint32_t)kmax : 0u, N = kmin < 0 ? (uint32_t)(-kmin) : 0u;
    const int cpos = P >= 1 ? 32 + bit_length_u32(P) : NO_CANDIDATE;          // one too many if P 2^32 itself is the largest
    const int cneg = N >= 2 ? 32 + bit_length_u32(N - 1u) : NO_CANDIDATE;
    needs_exact = P >= 1 ? ((P & (P - 1u)) == 0 && cpos > cneg) : N <= 1;
    const int c = cpos > cneg ? cpos : cneg;
    return unit - F + c;
}
OZAKI_SLICE_HD int narrow_candidate_exact(uint64_t max_abs, int unit, int F) {
    if (max_abs == 0) return NO_CANDIDATE;
    return unit - F + bit_length_u64(max_abs) - (((max_abs & (max_abs - 1)) == 0) ? 1 : 0);
}

}  // namespace ozaki
