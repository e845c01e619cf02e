/*
 * IEEE binary64 multiplication written out from its definition, with integer arithmetic only
 * (oracle; test infrastructure -- never linked into the product library).
 *
 * The paper's Section 4.2 emulates the FP64 multiplication with 32/64-bit integer operations
 * (its listing shows the 64 x 64 -> 128 bit product of the two significands assembled from four
 * 32 x 32 bit partial products), rounding to nearest-even, bitwise identical to the hardware
 * result, without overflow, underflow and subnormal handling.  This file is the "definition"
 * form: the exact product of the two 53-bit significands as one 128-bit integer, rounded once
 * to 53 bits (ties to even), exponents added.
 *
 * Operands and results must be zeros or normal numbers; a result that would leave the normal
 * range is returned as a zero / infinity of the right sign.
 */
#include <stdint.h>
#include <stddef.h>

typedef unsigned __int128 u128;

uint64_t oracle_fp64_mul_bits(uint64_t a, uint64_t b)
{
    const uint64_t SIGN = 0x8000000000000000ull;
    const uint64_t FRAC = 0x000FFFFFFFFFFFFFull;
    uint64_t s = (a ^ b) & SIGN;
    int ea = (int)((a >> 52) & 0x7FF), eb = (int)((b >> 52) & 0x7FF);
    if (ea == 0 || eb == 0) return s;                      /* zero (or subnormal: outside the contract) */

    uint64_t ma = (a & FRAC) | (1ull << 52), mb = (b & FRAC) | (1ull << 52);
    u128 prod = (u128)ma * (u128)mb;                       /* in [2^104, 2^106) */
    int e = ea + eb - 1023;                                /* biased exponent if the product lies in [2^104, 2^105) */
    int sh = 52;                                           /* bits to drop so that 53 remain */
    if (prod >> 105) { sh = 53; e += 1; }
    u128 kept = prod >> sh;
    u128 rem = prod & (((u128)1 << sh) - 1);
    u128 half = (u128)1 << (sh - 1);
    if (rem > half || (rem == half && (kept & 1))) kept += 1;
    if (kept >> 53) { kept >>= 1; e += 1; }                /* rounding carried into a new binade */
    if (e >= 0x7FF) return s | 0x7FF0000000000000ull;
    if (e <= 0) return s;
    return s | ((uint64_t)e << 52) | ((uint64_t)kept & FRAC);
}

void oracle_fp64_mul_array(const uint64_t* a, const uint64_t* b, uint64_t* out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = oracle_fp64_mul_bits(a[i], b[i]);
}
