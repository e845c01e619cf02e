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
void host_int32_scaled_to_fp64(const int* v, const int* e2, uint64_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = ozaki::int32_scaled_to_fp64(v[i], e2[i]);
}
void host_fp64_scale_pow2(const uint64_t* x, const int* e2, uint64_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = ozaki::fp64_scale_pow2_emulated(x[i], e2[i]);
}
}
