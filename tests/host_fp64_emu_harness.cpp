// Host build of the product's integer-only FP64 routines, for CPU-side unit tests (no GPU involved).
#include "../paper_2508_00441_amd/csrc/fp64_emu.hpp"
#include <stddef.h>

extern "C" {
void host_fp64_add_emulated(const uint64_t* a, const uint64_t* b, uint64_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = ozaki::fp64_add_emulated(a[i], b[i]);
}
void host_fp64_mul_emulated(const uint64_t* a, const uint64_t* b, uint64_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = ozaki::fp64_mul_emulated(a[i], b[i]);
}
void host_mul_64x64_128(const uint64_t* a, const uint64_t* b, uint64_t* hi, uint64_t* lo, size_t n) {
    for (size_t i = 0; i < n; ++i) ozaki::mul_64x64_128(a[i], b[i], hi[i], lo[i]);
}
void host_int53_scaled_to_fp64(const int64_t* v, const int* e2, uint64_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = ozaki::int53_scaled_to_fp64(v[i], e2[i]);
}
// n_seq sequences of len terms v * 2^e2 each, summed front to back with ozaki::RoundedSum; start[i] != 0 begins
// from those FP64 bits instead of zero.  exact_adds counts the additions done on integers.
void host_rounded_sum(const int64_t* v, const int* e2, const uint64_t* start, uint64_t* out, long long* exact_adds, size_t n_seq, size_t len) {
    long long cnt = 0;
    for (size_t i = 0; i < n_seq; ++i) {
        ozaki::RoundedSum s;
        if (start[i]) s.start_at(start[i]); else s.start_at_zero();
        for (size_t j = 0; j < len; ++j) {
            cnt += s.add(v[i * len + j], e2[i * len + j]);
        }
        out[i] = s.value();
    }
    *exact_adds = cnt;
}
// n_seq sequences of len terms v * 2^sh (sh may be negative: cut towards minus infinity) summed in ozaki::Fixed192;
// out_words: the three words of each sum; out_fp64: the sum times 2^unit_e2[i] rounded once.
void host_fixed192(const int64_t* v, const int* sh, const int* unit_e2, uint64_t* out_words, uint64_t* out_fp64, size_t n_seq, size_t len) {
    for (size_t i = 0; i < n_seq; ++i) {
        ozaki::Fixed192 x;
        x.clear();
        for (size_t j = 0; j < len; ++j) x.add(v[i * len + j], sh[i * len + j]);
        out_words[3 * i] = x.w0; out_words[3 * i + 1] = x.w1; out_words[3 * i + 2] = x.w2;
        out_fp64[i] = x.round_to_fp64(unit_e2[i]);
    }
}
void host_fp64_scale_pow2(const uint64_t* x, const int* e2, uint64_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = ozaki::fp64_scale_pow2_emulated(x[i], e2[i]);
}
}
