/*
 * IEEE binary64 addition written out from its definition, with integer arithmetic only
 * (oracle; test infrastructure -- never linked into the product library).
 *
 * The paper's Section 4.2 replaces the FP64 additions of the accumulation step by an
 * emulation built on 32/64-bit integer operations that rounds to nearest-even and is
 * bitwise identical to the hardware result, leaving out overflow, underflow and
 * subnormal numbers.  This file is the "definition" form of that operation:
 *
 *   1. decode both operands into sign, exponent, 53-bit significand;
 *   2. place both significands exactly on a common fixed-point grid (128-bit integer);
 *      an operand more than 64 binades below the other cannot change the rounded
 *      result and is dropped (see the comment at the cut-off);
 *   3. add the signed integers exactly;
 *   4. round the exact result once to 53 bits, ties to even; re-encode.
 *
 * Operands and results must be zeros or normal numbers; a result that would leave the
 * normal range is returned as a zero / infinity of the right sign (the paper omits
 * these cases; the tests stay inside the normal range).
 */
#include <stdint.h>
#include <stddef.h>

typedef unsigned __int128 u128;

static int top_bit(u128 v)            /* index of the highest set bit, v != 0 */
{
    int n = -1;
    while (v) { v >>= 1; ++n; }
    return n;
}

uint64_t oracle_fp64_add_bits(uint64_t a, uint64_t b)
{
    const uint64_t SIGN = 0x8000000000000000ull;
    const uint64_t FRAC = 0x000FFFFFFFFFFFFFull;
    int ea = (int)((a >> 52) & 0x7FF), eb = (int)((b >> 52) & 0x7FF);

    /* zeros (subnormals are treated as zeros: outside the emulation's contract) */
    if (ea == 0 && eb == 0) return (a & b & SIGN);         /* (+0)+(-0) = +0, (-0)+(-0) = -0 */
    if (ea == 0) return b;
    if (eb == 0) return a;

    /* order by magnitude: |a| >= |b| */
    if ((a & ~SIGN) < (b & ~SIGN)) { uint64_t t = a; a = b; b = t; int te = ea; ea = eb; eb = te; }
    int d = ea - eb;
    /* A non-zero addend of magnitude below ulp(a)/2^11 can only move the exact sum strictly
       inside the rounding interval of a (even when a is a power of two and the addend has the
       opposite sign, where the interval's lower half-width is ulp/4), so the result is a. */
    if (d > 64) return a;

    uint64_t ma = (a & FRAC) | (1ull << 52), mb = (b & FRAC) | (1ull << 52);
    int neg_a = (a & SIGN) != 0, neg_b = (b & SIGN) != 0;

    /* common grid: unit = 2^(eb - 1075); |a| = ma << d, |b| = mb */
    u128 big = (u128)ma << d, small = (u128)mb, mag;
    int neg;
    if (neg_a == neg_b) { mag = big + small; neg = neg_a; }
    else                { mag = big - small; neg = neg_a; }  /* big >= small by the ordering */
    if (mag == 0) return 0;                                   /* exact cancellation: +0 under round-to-nearest */

    /* one rounding to 53 bits, ties to even */
    int tb = top_bit(mag);
    int e = eb + (tb - 52);                                   /* biased exponent of the leading bit */
    uint64_t sig;
    if (tb <= 52) {
        sig = (uint64_t)(mag << (52 - tb));                   /* exact */
    } else {
        int sh = tb - 52;
        u128 kept = mag >> sh;
        u128 rem = mag & (((u128)1 << sh) - 1);
        u128 half = (u128)1 << (sh - 1);
        if (rem > half || (rem == half && (kept & 1))) kept += 1;
        if (kept >> 53) { kept >>= 1; e += 1; }               /* rounding carried into a new binade */
        sig = (uint64_t)kept;
    }
    uint64_t s = neg ? SIGN : 0;
    if (e >= 0x7FF) return s | 0x7FF0000000000000ull;
    if (e <= 0) return s;
    return s | ((uint64_t)e << 52) | (sig & FRAC);
}

/* out[i] = a[i] (+) b[i] on raw bit patterns */
void oracle_fp64_add_array(const uint64_t *a, const uint64_t *b, uint64_t *out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = oracle_fp64_add_bits(a[i], b[i]);
}
