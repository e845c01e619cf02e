// Host build of the slicer's per-element routines, for CPU-side unit tests (no GPU involved): one vector is
// sliced the way the kernel does it, with "threads" of `chunk` consecutive elements that each form their own
// candidate for the next exponent.
#include "../paper_2508_00441_amd/csrc/slice_element.hpp"
#include <stddef.h>
#include <vector>

extern "C" {
// x: n FP64 bit patterns.  q_out: [s][n] slice integers, c_out: [s] exponents.  Returns 2 * (number of times the lower
// upper words could not decide a thread's candidate) + (1 if a non-finite input was seen).
int host_slice_vector_narrow(const uint64_t* x, size_t n, int b, int s, int chunk, int* q_out, int* c_out) {
    using namespace ozaki;
    const int F = 60 - b, pos = F - 32, bias = (1 << (pos - 1)) - 1;
    const uint32_t keep = ~((1u << pos) - 1u);
    std::vector<int> pk(n);
    std::vector<uint64_t> T(n);
    bool nonfinite = false;
    int cmax = NO_CANDIDATE;
    for (size_t i = 0; i < n; ++i) decode_narrow(x[i], F, T[i], pk[i], cmax, nonfinite);
    int unit_prev = 0, low_decisions = 0;
    std::vector<char> all_active((n + chunk - 1) / chunk + 1, 0);     // per thread: no element waits any more
    for (int p = 0; p < s; ++p) {
        const int c = cmax == NO_CANDIDATE ? 0 : cmax;
        const int unit = c - b;
        const int step16 = (unit_prev - unit) * 65536;
        unit_prev = unit;
        c_out[p] = c;
        int next = NO_CANDIDATE;
        for (size_t i0 = 0, th = 0; i0 < n; i0 += chunk, ++th) {
            const size_t i1 = i0 + chunk < n ? i0 + chunk : n;
            int kmax = KEY_NONE_MAX, kmin = KEY_NONE_MIN;
            uint32_t cd_wait = 0;
            if (all_active[th]) {
                for (size_t i = i0; i < i1; ++i)
                    q_out[(size_t)p * n + i] = slice_narrow_active(T[i], step16 / 65536, pos, bias, keep, kmax, kmin) >> pos;
            } else {
                for (size_t i = i0; i < i1; ++i)
                    q_out[(size_t)p * n + i] = slice_narrow(T[i], pk[i], step16, pos, bias, keep, kmax, kmin, cd_wait) >> pos;
                all_active[th] = cd_wait == 0;
            }
            bool needs_exact;
            int cand = narrow_candidate(kmax, kmin, unit, F, needs_exact);
            if (needs_exact) {
                ++low_decisions;
                uint64_t mx = 0;
                for (size_t i = i0; i < i1; ++i) {
                    const uint64_t a = (all_active[th] || pk[i] == 0) ? narrow_abs(T[i]) : 0u;
                    mx = a > mx ? a : mx;
                }
                cand = narrow_candidate_exact(mx, unit, F);
            }
            if (cd_wait != 0 && (int)cd_wait - CD_BIAS > cand) cand = (int)cd_wait - CD_BIAS;
            next = cand > next ? cand : next;
        }
        cmax = next;
    }
    return 2 * low_decisions + (nonfinite ? 1 : 0);
}
}
