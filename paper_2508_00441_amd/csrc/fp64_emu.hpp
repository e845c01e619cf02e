// IEEE binary64 addition and multiplication with 32/64-bit integer instructions only (paper Section 4.2).
//
// Round-to-nearest-even, bitwise equal to a hardware FP64 add for operands and results that are
// zeros or normal numbers.  As in the paper, overflow, underflow and subnormal numbers are not
// handled: a result below the normal range is flushed to a signed zero, one above it becomes a
// signed infinity, and subnormal operands are treated as zeros.
//
// The significands carry three extra low bits (guard, round, sticky); that is enough because an
// effective subtraction either has an exponent difference <= 1 (then it is exact and may need a
// long normalisation shift) or needs at most a one-bit normalisation shift.
//
// The header compiles for the device (hipcc) and, for CPU-side unit tests of this very code, for the
// host (any C++ compiler): OZAKI_HD expands to nothing there.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define OZAKI_HD __host__ __device__ __forceinline__
#else
#define OZAKI_HD inline
#endif

namespace ozaki {

OZAKI_HD int clz64(uint64_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __clzll((long long)v);
#else
    return __builtin_clzll(v);
#endif
}

constexpr uint64_t F64_SIGN = 0x8000000000000000ull;
constexpr uint64_t F64_FRAC = 0x000FFFFFFFFFFFFFull;
constexpr uint64_t F64_HIDDEN = 0x0010000000000000ull;
constexpr uint64_t F64_INF = 0x7FF0000000000000ull;

// a (+) b on raw bit patterns.
OZAKI_HD uint64_t fp64_add_emulated(uint64_t a, uint64_t b) {
    uint64_t abs_a = a & ~F64_SIGN, abs_b = b & ~F64_SIGN;
    // Zeros (and subnormals, by contract): x + 0 = x; (+0) + (-0) = +0.
    if (abs_b < F64_HIDDEN) return (abs_a < F64_HIDDEN) ? (a & b & F64_SIGN) : a;
    if (abs_a < F64_HIDDEN) return b;
    if (abs_a < abs_b) {                       // order by magnitude
        uint64_t t = a; a = b; b = t;
        t = abs_a; abs_a = abs_b; abs_b = t;
    }
    int e = (int)(abs_a >> 52);
    int d = e - (int)(abs_b >> 52);
    uint64_t ma = ((abs_a & F64_FRAC) | F64_HIDDEN) << 3;    // hidden bit at position 55
    uint64_t mb = ((abs_b & F64_FRAC) | F64_HIDDEN) << 3;
    if (d > 0) {
        if (d >= 57) {
            mb = 1;                                            // pure sticky
        } else {
            uint64_t lost = mb & ((1ull << d) - 1);
            mb = (mb >> d) | (lost != 0);
        }
    }
    uint64_t sign = a & F64_SIGN;
    uint64_t m;
    if ((a ^ b) & F64_SIGN) {
        m = ma - mb;
        if (m == 0) return 0;                                  // exact cancellation gives +0
        int lz = clz64(m) - 8;                                 // bring the leading bit back to position 55
        m <<= lz;
        e -= lz;
    } else {
        m = ma + mb;
        if (m >> 56) {                                         // carry out: one step right, keep the sticky bit
            m = (m >> 1) | (m & 1);
            e += 1;
        }
    }
    uint64_t sig = m >> 3;                                     // 53 bits, hidden bit at position 52
    unsigned grs = (unsigned)m & 7u;
    sig += (grs > 4u) | ((grs == 4u) & (unsigned)(sig & 1));   // ties to even; a carry to 2^53 is absorbed below
    if (e <= 0) return sign;
    uint64_t r = ((uint64_t)e << 52) + (sig - F64_HIDDEN);     // sig == 2^53 bumps the exponent, fraction 0
    if (r >= F64_INF) return sign | F64_INF;
    return sign | r;
}

// Full 64 x 64 -> 128 bit product from four 32 x 32 -> 64 bit partial products (the pen-and-paper scheme with
// 32-bit digits of Section 4.2).  The middle column is summed in a way that cannot overflow: three terms below 2^32.
OZAKI_HD void mul_64x64_128(uint64_t x, uint64_t y, uint64_t& hi, uint64_t& lo) {
    const uint64_t x0 = (uint32_t)x, x1 = x >> 32, y0 = (uint32_t)y, y1 = y >> 32;
    const uint64_t p00 = x0 * y0, p01 = x0 * y1, p10 = x1 * y0, p11 = x1 * y1;
    const uint64_t mid = (p00 >> 32) + (uint32_t)p01 + (uint32_t)p10;
    lo = (mid << 32) | (uint32_t)p00;
    hi = p11 + (p01 >> 32) + (p10 >> 32) + (mid >> 32);
}

// a (x) b on raw bit patterns: IEEE binary64 multiplication, round-to-nearest-even, for zeros and normal numbers
// (same contract as the addition above).
OZAKI_HD uint64_t fp64_mul_emulated(uint64_t a, uint64_t b) {
    const uint64_t sign = (a ^ b) & F64_SIGN;
    const int ea = (int)((a >> 52) & 0x7FF), eb = (int)((b >> 52) & 0x7FF);
    if (ea == 0 || eb == 0) return sign;
    // significands scaled by 2^5 and 2^6: the 106-bit product scaled by 2^11 has its leading bit at position 116 or
    // 115, so the upper word holds 53 or 52 significant bits and the lower word all the bits below them
    const uint64_t ma = ((a & F64_FRAC) | F64_HIDDEN) << 5, mb = ((b & F64_FRAC) | F64_HIDDEN) << 6;
    uint64_t hi, lo;
    mul_64x64_128(ma, mb, hi, lo);
    int e = ea + eb - 1023;
    if (hi >> 52) {
        e += 1;                                                // product of the significands in [2, 4)
    } else {
        hi = (hi << 1) | (lo >> 63);                           // in [1, 2): one more bit from below
        lo <<= 1;
    }
    const uint64_t half = 0x8000000000000000ull;
    hi += (uint64_t)((lo > half) | ((lo == half) & (unsigned)(hi & 1)));     // ties to even
    if (e <= 0) return sign;
    const uint64_t r = ((uint64_t)e << 52) + (hi - F64_HIDDEN);               // hi == 2^53 bumps the exponent
    if (r >= F64_INF) return sign | F64_INF;
    return sign | r;
}

// n * 2^e2 as FP64 bits for an integer |n| <= 2^53 (exact), integer-only; flushed / saturated outside the normal range.
OZAKI_HD uint64_t int53_scaled_to_fp64(int64_t n, int e2) {
    if (n == 0) return 0;
    const uint64_t sign = n < 0 ? F64_SIGN : 0;
    const uint64_t a = (uint64_t)(n < 0 ? -n : n);
    const int top = 63 - clz64(a);                           // position of the leading one
    const int e = 1023 + top + e2;
    if (e <= 0) return sign;
    if (e >= 2047) return sign | F64_INF;
    const uint64_t sig = top <= 52 ? a << (52 - top) : a >> 1;     // top == 53 only for 2^53 itself
    return sign | ((uint64_t)e << 52) | (sig & F64_FRAC);
}

// A running FP64 sum of terms v * 2^e2 (v an integer below 2^52 in magnitude), each addition rounded to nearest even.
// The sum is held as x * 2^ex with a 64-bit integer |x| <= 2^53: an FP64 value written with an unnormalised
// significand.  When both operands fit one 64-bit integer in units of the smaller of their two scales (the usual
// case: the method's terms arrive least significant first, a few bits apart), the addition is an integer addition
// followed by one rounding of the result to 53 significant bits, ties to even -- what the IEEE addition returns,
// and nothing at all while the result is short enough to be exact.  A term that towers over the sum is handled the same
// way after the sum has been cut down to the term's scale with a sticky bit; only a term far below the sum's unit (the
// method does not produce one) goes through fp64_add_emulated.  Bit for bit the chain of rounded additions, inside the
// normal range.
struct RoundedSum {
    int64_t x;
    int ex;

    OZAKI_HD void start_at_zero() { x = 0; ex = 0; }
    OZAKI_HD void start_at(uint64_t fp64_bits) {
        const int e = (int)((fp64_bits >> 52) & 0x7FF);
        const int64_t m = (int64_t)((fp64_bits & F64_FRAC) | F64_HIDDEN);
        x = e == 0 ? 0 : (fp64_bits & F64_SIGN) ? -m : m;
        ex = e - 1075;
    }
    // Returns whether the addition was done on integers (false: the general routine was needed).
    OZAKI_HD bool add(int64_t v, int e2) {
        if (v == 0) return true;                                // adding an exact zero changes nothing
        const uint64_t sv = (uint64_t)(v >> 63);
        return add_bits(v, e2, 64 - clz64(((uint64_t)v ^ sv) - sv));
    }
    OZAKI_HD bool add(int v, int e2) {                          // same for a 32-bit term: cheaper bit count
        if (v == 0) return true;
        const uint32_t av = (uint32_t)(v < 0 ? -v : v);
#if defined(__HIP_DEVICE_COMPILE__)
        return add_bits((int64_t)v, e2, 32 - __clz((int)av));
#else
        return add_bits((int64_t)v, e2, 32 - __builtin_clz(av));
#endif
    }
    // v != 0 with nv significant bits
    OZAKI_HD bool add_bits(int64_t v, int e2, int nv) {
        if (x == 0) { x = v; ex = e2; return true; }            // keeps the term's own (low) unit: the sum stays short for long
        const int d = e2 - ex;
        if (d < -8) {                                           // the term lies far below the sum's unit: general routine
            start_at(fp64_add_emulated(int53_scaled_to_fp64(x, ex), int53_scaled_to_fp64(v, e2)));
            return false;
        }
        int64_t t;
        int e = ex;
        if (nv + d <= 62) {                                     // |x| << 8 and |v| << d both stay below 2^62
            if (d >= 0) {                                       // the usual case: the term's unit is not below the sum's
                t = (int64_t)((uint64_t)x + ((uint64_t)v << d));
            } else {
                t = (int64_t)(((uint64_t)x << -d) + (uint64_t)v);
                e = e2;
            }
        } else {
            // The term towers over the sum: bring the term's leading bit to position 61 and the sum down to that unit,
            // by r >= 1 bits; what the sum loses is kept as a set lowest bit.  The result then has at least 60 bits,
            // at least 7 are dropped, and an odd integer is never a tie or a 53-bit number at that cut, so the
            // rounding below sees the same side of every boundary as the exact sum does.
            const int up = 62 - nv, r = d - up;                 // r = nv + d - 62 > 0
            const uint64_t sx = (uint64_t)(x >> 63);
            const uint64_t ax = ((uint64_t)x ^ sx) - sx;
            const uint64_t kept = r < 64 ? ax >> r : 0;
            const uint64_t lost = r < 64 ? ax & ((1ull << r) - 1) : ax;
            const uint64_t xs = kept | (lost != 0 ? 1u : 0u);
            t = (int64_t)(((uint64_t)v << up) + ((xs ^ sx) - sx));
            e = e2 - up;
        }
        // Round t to 53 significant bits, ties to even, on the two's-complement number itself.  The bit count is
        // taken from t with its bits flipped if negative (|t| - 1): that is the bit count of |t| except for a negative
        // power of two, which then keeps one bit more -- it is exact either way and stays within |x| <= 2^53.
        const uint64_t flipped = (uint64_t)(t ^ (t >> 63));
        const int drop = 11 - clz64(flipped | 1);               // bits beyond 53
        if (drop > 0) {
            x = (t + (((int64_t)1 << (drop - 1)) - 1) + ((t >> drop) & 1)) >> drop;      // may reach +-2^53
            ex = e + drop;
        } else {
            x = t;
            ex = e;
        }
        return true;
    }
    OZAKI_HD uint64_t value() const { return int53_scaled_to_fp64(x, ex); }
};

// A 192-bit two's-complement fixed-point accumulator: the exact sum of terms v * 2^sh units (v an integer of at most
// 2^36 in magnitude, sh <= 144), rounded to FP64 once at the end.  1024 such terms stay below 2^190: no overflow.
struct Fixed192 {
    uint64_t w0, w1, w2;                                        // least significant word first

    OZAKI_HD void clear() { w0 = w1 = w2 = 0; }
    // += v * 2^sh.  A negative sh cuts the term to whole units towards minus infinity (arithmetic shift).
    OZAKI_HD void add(int64_t v, int sh) {
        if (sh < 0) {
            v >>= (sh < -63 ? 63 : -sh);
            sh = 0;
        }
        const int word = sh >> 6, bit = sh & 63;
        const uint64_t lo = (uint64_t)v << bit;
        const uint64_t hi = (uint64_t)((v >> 1) >> (63 - bit));      // bits 64.. of the shifted value, sign-extended
        const uint64_t ext = (uint64_t)(v >> 63);                    // all sign bits
        // the addend as three words, placed by the word index without branching
        const uint64_t a0 = word == 0 ? lo : 0;
        const uint64_t a1 = word == 0 ? hi : word == 1 ? lo : 0;
        const uint64_t a2 = word == 0 ? ext : word == 1 ? hi : lo;
        const uint64_t s0 = w0 + a0;
        const uint64_t c0 = s0 < a0;
        const uint64_t t1 = w1 + a1;
        const uint64_t c1 = t1 < a1;
        const uint64_t s1 = t1 + c0;
        const uint64_t c1b = s1 < c0;
        w0 = s0;
        w1 = s1;
        w2 = w2 + a2 + c1 + c1b;
    }
    // The sum times 2^unit_e2, rounded to the nearest FP64 value, ties to even; flushed / saturated outside the normal
    // range like the other routines of this header.
    OZAKI_HD uint64_t round_to_fp64(int unit_e2) const {
        uint64_t m0 = w0, m1 = w1, m2 = w2;
        const uint64_t sign = m2 & F64_SIGN;
        if (sign) {                                                 // magnitude = two's complement negation
            m0 = ~m0 + 1;
            const uint64_t c = m0 == 0;
            m1 = ~m1 + c;
            m2 = ~m2 + ((c != 0 && m1 == 0) ? 1 : 0);
        }
        if ((m0 | m1 | m2) == 0) return 0;
        const int top = m2 ? 191 - clz64(m2) : m1 ? 127 - clz64(m1) : 63 - clz64(m0);     // leading one
        uint64_t sig;
        if (top <= 52) {
            sig = m0 << (52 - top);                                 // short enough: exact
        } else {
            // the 55 bits from the leading one down (53 of the significand, a guard bit, one more), then sticky
            const int r = top - 54;                                 // bits below those 55; may be negative (top 53, 54)
            uint64_t head;
            bool sticky;
            if (r <= 0) {
                head = m0 << (-r);
                sticky = false;
            } else {
                const int word = r >> 6, bit = r & 63;
                const uint64_t x0 = word == 0 ? m0 : word == 1 ? m1 : m2;
                const uint64_t x1 = word == 0 ? m1 : word == 1 ? m2 : 0;
                head = bit ? (x0 >> bit) | (x1 << (64 - bit)) : x0;
                const uint64_t below = bit ? (x0 << (64 - bit)) : 0;
                sticky = below != 0 || (word >= 1 && m0 != 0) || (word == 2 && m1 != 0);
            }
            sig = head >> 2;                                        // 53 bits, leading one at position 52
            const unsigned guard = (unsigned)(head >> 1) & 1u, rest = ((unsigned)head & 1u) | (sticky ? 1u : 0u);
            sig += guard & (rest | (unsigned)(sig & 1));            // a carry to 2^53 bumps the exponent below
        }
        const int e = 1023 + top + unit_e2;
        if (e <= 0) return sign;
        const uint64_t rbits = ((uint64_t)e << 52) + (sig - F64_HIDDEN);
        if (rbits >= F64_INF) return sign | F64_INF;
        return sign | rbits;
    }
};

// x * 2^e2 on FP64 bits (zeros stay zeros; the result is flushed / saturated outside the normal range).
OZAKI_HD uint64_t fp64_scale_pow2_emulated(uint64_t x, int e2) {
    uint64_t ax = x & ~F64_SIGN;
    if (ax < F64_HIDDEN) return x & F64_SIGN;
    int e = (int)(ax >> 52) + e2;
    if (e <= 0) return x & F64_SIGN;
    if (e >= 2047) return (x & F64_SIGN) | F64_INF;
    return (x & (F64_SIGN | F64_FRAC)) | ((uint64_t)e << 52);
}

}  // namespace ozaki
